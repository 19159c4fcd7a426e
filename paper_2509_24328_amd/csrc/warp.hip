// sv_warp_cutoffs: per-row cutoff of the sampling warps temperature -> top-k ->
// top-p (the sampling hyper-parameters of the SV paper's appendix table), so
// that the warped distribution is soft-max(z / T) restricted to {v : z_v >= cutoff}.
// Entries of equal value are kept or dropped together.
//
// One workgroup per row.  Both warps only concern the upper tail of the row, so
// the kernel first tries to settle them on a short list of candidates:
//   sweep 1  per-lane online (max, sum-exp): row maximum m, normaliser Z, bad-row
//            detection; the 512 lane maxima are distinct entries of the row, so the
//            K-th largest of them is a lower bound of the K-th largest entry
//   select   tau = that bound (top-k), or the 384-th largest lane maximum (top-p
//            alone: a guess that leaves a few hundred to a few thousand candidates)
//   sweep 2  (from cache) append every entry >= tau to a list in LDS
//   settle   sort the list, read off the K-th largest value, walk the groups of equal
//            value until their mass reaches P
// The list is exact whenever it holds at least K entries and (top-p alone) at
// least P of the row's mass.  Otherwise - flat rows, huge K, more than 2048
// candidates - the general path takes over: radix selection on an order-preserving
// 32-bit key of the logit (11 + 11 + 10 bits; bfloat16 rows are resolved after two
// levels), one histogram sweep of counts and masses per level.
// Masses are fp64 exponentials (candidate path; the row total of top-p alone comes
// from the fp32 sweep) or fp32 ones summed with LDS float atomics (general path); a
// top-p decision within 3e-6 of P is flagged SV_FLAG_NEAR_TIE.
//
// sv_warp_compact is the same kernel with one more step: the kept entries of a
// settled list are the whole support of the warped distribution, so their token
// ids (ascending) and fp64 probabilities are written out and everything
// downstream can work on a few dozen entries per row instead of V.
#include "sv_device.hpp"
#include "sv_host.hpp"

namespace sv {

constexpr int kWarpThreads = 512;
constexpr int kBins = 2048;
constexpr int kCand = 2048;          // capacity of the candidate list
constexpr int kGuessRank = 384;      // top-p alone: tau = this rank among the lane maxima
constexpr double kNearTie = 3e-6;    // flagged band of a top-p decision

__device__ __forceinline__ uint32_t okey(float f) {            // ascending order-preserving key
  const uint32_t u = __float_as_uint(f);
  return (u >> 31) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float from_okey(uint32_t k) {
  return __uint_as_float((k >> 31) ? (k & 0x7fffffffu) : ~k);
}

// digit of `key` at `level`, and whether the key lies under `prefix` (the
// digits of the levels above)
__device__ __forceinline__ int level_shift(int level) { return level == 0 ? 21 : (level == 1 ? 10 : 0); }
__device__ __forceinline__ int level_bits(int level) { return level == 2 ? 10 : 11; }
__device__ __forceinline__ uint32_t digit_of(uint32_t key, int level) {
  return (key >> level_shift(level)) & ((1u << level_bits(level)) - 1u);
}
__device__ __forceinline__ bool under_prefix(uint32_t key, uint32_t prefix, int level) {
  return level == 0 || (key >> (level_shift(level) + level_bits(level))) == prefix;
}

struct alignas(16) WarpShared {
  BlockScratch red;
  MergeScratch<1> mg;
  union {
    struct {                   // general path
      uint32_t cnt[kBins];
      float mass[kBins];
      float mass0[kBins];      // level-0 masses, kept for the top-p pass
    };
    struct {                   // candidate path
      uint64_t key[kCand];     // (order key of the value, ~token id): sorted descending
      double w[kCand];         // masses exp((z - m) / T) of the sorted candidates
      float lane_max[kWarpThreads];
    };
  };
  float tau, theta;
  int n_cand, settled, n_keep;
  double z_keep;               // mass of the kept entries
  int sel_digit;
  uint32_t sel_count_above;
  double sel_mass_above;
  double sel_mass_bin;
  int near_tie;
};

// Scan the histograms from the top digit down.  by_count: find the digit where
// the cumulative count reaches `k_rem`; else where the cumulative mass reaches
// `target`.  One lane; results in LDS.
__device__ __forceinline__ void scan_bins(WarpShared& sh, int nbins, bool by_count, uint32_t k_rem, double target,
                                          double total_for_tie) {
  uint32_t c_above = 0;
  double m_above = 0.0;
  int found = 0;
  for (int d = nbins - 1; d >= 0; --d) {
    const uint32_t c = sh.cnt[d];
    const double mm = (double)sh.mass[d];
    const bool hit = by_count ? (c_above + c >= k_rem) : (m_above + mm >= target && c > 0);
    if (!by_count && c > 0 && total_for_tie > 0.0) {
      // the candidate group boundaries at this level: flag a decision that sits on P
      const double fr = (m_above + mm) / total_for_tie, want = target / total_for_tie;
      if (fabs(fr - want) < kNearTie) sh.near_tie = 1;
    }
    if (hit || d == 0) { found = d; sh.sel_mass_bin = mm; break; }
    c_above += c;
    m_above += mm;
  }
  sh.sel_digit = found;
  sh.sel_count_above = c_above;
  sh.sel_mass_above = m_above;
}

// General path: radix selection over the whole row (m = row maximum, finite).
// Returns the cutoff in every thread; sets sh.near_tie.
template <int DT>
__device__ __noinline__ float general_cutoff(const void* row, int V, float lt, int top_k, float top_p, float m,
                                             WarpShared& sh) {
  const int tid = threadIdx.x;
  constexpr int kLevels = (DT == DT_BF16) ? 2 : 3;
  const bool use_k = top_k > 0 && top_k < V, use_p = top_p < 1.0f;
  const float c_ref = m * lt;

  // histogram sweep over the entries under `prefix` at `level`, optionally only z >= floor_v
  auto histogram = [&](int level, uint32_t prefix, float floor_v) {
    for (int d = tid; d < kBins; d += blockDim.x) { sh.cnt[d] = 0; sh.mass[d] = 0.f; }
    __syncthreads();
    visit_range<DT, false, 4>(row, nullptr, 0, V, [&](int, float v, float) {
      const uint32_t key = okey(v);
      if (under_prefix(key, prefix, level) && v >= floor_v) {
        const uint32_t d = digit_of(key, level);
        atomicAdd(&sh.cnt[d], 1u);
        atomicAdd(&sh.mass[d], exp2_fast(__builtin_fmaf(v, lt, -c_ref)));
      }
    });
    __syncthreads();
  };

  // sweep 2: level 0 over everything
  histogram(0, 0u, -INFINITY);
  for (int d = tid; d < kBins; d += blockDim.x) sh.mass0[d] = sh.mass[d];
  double total0 = 0.0;
  {
    double part = 0.0;
    for (int d = tid; d < kBins; d += blockDim.x) part += (double)sh.mass[d];
    total0 = block_sum_f64(part, sh.red);
  }

  // ---- top-k: K-th largest value ------------------------------------------
  float t_k = -INFINITY;
  double total_k = total0;
  int dk0 = -1;                       // level-0 digit of t_k
  double surv_in_dk0 = 0.0;           // mass of the survivors inside that digit
  if (use_k) {
    uint32_t prefix = 0, k_rem = (uint32_t)top_k;
    double mass_above = 0.0, mass_above_l0 = 0.0;
    for (int level = 0; level < kLevels; ++level) {
      if (level > 0) histogram(level, prefix, -INFINITY);
      if (tid == 0) scan_bins(sh, 1 << level_bits(level), true, k_rem, 0.0, 0.0);
      __syncthreads();
      const int d = sh.sel_digit;
      k_rem -= sh.sel_count_above;
      mass_above += sh.sel_mass_above;
      if (level == 0) { dk0 = d; mass_above_l0 = sh.sel_mass_above; }
      prefix = (prefix << level_bits(level)) | (uint32_t)d;
      if (level == kLevels - 1) total_k = mass_above + sh.sel_mass_bin;
      __syncthreads();
    }
    // bfloat16: the ten low key bits are all ones for negative values, zero otherwise
    const uint32_t key = (DT == DT_BF16) ? ((prefix << 10) | ((prefix >> 21) ? 0u : 0x3ffu)) : prefix;
    t_k = from_okey(key);
    surv_in_dk0 = total_k - mass_above_l0;
  }

  // ---- top-p over the survivors -------------------------------------------
  float theta = t_k;
  if (use_p) {
    const double target = (double)top_p * total_k;
    // level 0 from the saved masses: digits above dk0 survive whole, dk0 in part, below not at all
    for (int d = tid; d < kBins; d += blockDim.x) {
      float mm = sh.mass0[d];
      uint32_t c = mm > 0.f ? 1u : 0u;             // counts only mark non-empty bins here
      if (use_k) {
        if (d < dk0) { mm = 0.f; c = 0u; }
        else if (d == dk0) { mm = (float)surv_in_dk0; c = 1u; }
      }
      sh.mass[d] = mm;
      sh.cnt[d] = c;
    }
    __syncthreads();
    uint32_t prefix = 0;
    double acc = 0.0;
    for (int level = 0; level < kLevels; ++level) {
      if (level > 0) histogram(level, prefix, t_k);
      if (tid == 0) scan_bins(sh, 1 << level_bits(level), false, 0u, target - acc, level == kLevels - 1 ? total_k : 0.0);
      __syncthreads();
      acc += sh.sel_mass_above;
      prefix = (prefix << level_bits(level)) | (uint32_t)sh.sel_digit;
      __syncthreads();
    }
    const uint32_t key = (DT == DT_BF16) ? ((prefix << 10) | ((prefix >> 21) ? 0u : 0x3ffu)) : prefix;
    theta = fmaxf(from_okey(key), t_k);
  }
  return theta;
}

// Bitonic sort of c[0..n2) in descending order by the whole workgroup (n2 a power of two).
__device__ __forceinline__ void sort_desc(uint64_t* c, int n2) {
  const int tid = threadIdx.x, nt = blockDim.x;
  for (int k2 = 2; k2 <= n2; k2 <<= 1) {
    for (int j = k2 >> 1; j > 0; j >>= 1) {
      for (int i = tid; i < n2; i += nt) {
        const int o = i ^ j;
        if (o > i) {
          const uint64_t a = c[i], b = c[o];
          const bool desc = (i & k2) == 0;
          if (desc ? (a < b) : (a > b)) { c[i] = b; c[o] = a; }
        }
      }
      __syncthreads();
    }
  }
}

__device__ __forceinline__ float key_value(uint64_t key) { return from_okey((uint32_t)(key >> 32)); }
__device__ __forceinline__ uint32_t key_token(uint64_t key) { return 0xFFFFFFFFu - (uint32_t)key; }

// Optional outputs of sv_warp_compact (all null for sv_warp_cutoffs).
struct CompactOut {
  int32_t* count;    // [rows]
  int32_t* token;    // [rows, cap]
  double* prob;      // [rows, cap]
  float* lse;        // [rows]
  int cap;
};

template <int DT>
__global__ __launch_bounds__(kWarpThreads) void warp_cutoffs_kernel(const void* z, int V, Scale sc, int top_k,
                                                                    float top_p, float* cutoff, uint32_t* flags,
                                                                    CompactOut out) {
  __shared__ WarpShared sh;
  const int tid = threadIdx.x;
  const int r = blockIdx.x;
  const void* row = static_cast<const char*>(z) + (size_t)r * V * Elem<DT>::bytes;
  const float lt = sc.L;

  // sweep 1: maximum, normaliser, bad-row detection (NaN poisons the sum, +inf the maximum)
  Online acc[1];
  acc[0].init();
  sweep_online<DT, false, false>(row, V, 0, 1, acc[0], lt);
  MS merged[1];
  block_merge<1>(acc, sh.mg, merged, lt);
  const float m = merged[0].m;
  const double lse_row = lse_from_ms(merged[0], sc);   // of z / T over the whole row; NaN: bad row
  if (isnan(lse_row)) {
    if (tid == 0) {
      if (cutoff) cutoff[r] = __builtin_nanf("");
      if (flags) flags[r] = SV_FLAG_BAD_ROW;
      if (out.count) { out.count[r] = 0; out.lse[r] = __builtin_nanf(""); }
    }
    return;
  }
  const bool use_k = top_k > 0 && top_k < V, use_p = top_p < 1.0f;
  if (!use_k && !use_p && (V > kCand || !out.count)) {  // nothing to cut, and no short support to write
    if (tid == 0) {
      if (cutoff) cutoff[r] = -INFINITY;
      if (flags) flags[r] = 0;
      if (out.count) { out.count[r] = -1; out.lse[r] = (float)lse_row; }
    }
    return;
  }
  const double m_t = (double)m * sc.inv_t;
  const double Z = exp(lse_row - m_t);                  // sum_v exp((z_v - m) / T)

  // ---- candidate threshold from the lane maxima -----------------------------
  float tau = -INFINITY;                                // V <= kCand: every entry is a candidate
  bool try_list = true;
  if (V > kCand) {
    const int rank = use_k ? top_k : kGuessRank;       // tau = rank-th largest lane maximum
    if (rank > kWarpThreads) {
      try_list = false;
    } else {
      sh.lane_max[tid] = acc[0].m;
      if (tid == 0) sh.tau = -INFINITY;
      __syncthreads();
      const float mine = sh.lane_max[tid];
      int gt = 0, ge = 0;
      for (int j = 0; j < kWarpThreads; j += 4) {
        const float4 q = *reinterpret_cast<const float4*>(&sh.lane_max[j]);   // same address in all lanes
        gt += (q.x > mine) + (q.y > mine) + (q.z > mine) + (q.w > mine);
        ge += (q.x >= mine) + (q.y >= mine) + (q.z >= mine) + (q.w >= mine);
      }
      if (gt < rank && rank <= ge) sh.tau = mine;      // every lane that writes holds the same value
      __syncthreads();
      tau = sh.tau;
    }
  }

  float theta = 0.f;
  bool settled = false;
  if (tid == 0) { sh.n_cand = 0; sh.near_tie = 0; sh.settled = 0; sh.n_keep = -1; }
  __syncthreads();
  if (try_list) {
    // sweep 2: collect the candidates (a few per row: the shared counter is not a bottleneck)
    visit_range<DT, false, 4>(row, nullptr, 0, V, [&](int v, float zv, float) {
      if (zv >= tau && zv > -INFINITY) {                // entries at -inf carry no mass and are never listed
        const int at = atomicAdd(&sh.n_cand, 1);
        if (at < kCand) sh.key[at] = ((uint64_t)okey(zv) << 32) | (uint64_t)(0xFFFFFFFFu - (uint32_t)v);
      }
    });
    __syncthreads();
    const int n = sh.n_cand;
    // fewer than K candidates happens only when tau = -inf lists every finite entry
    // of the row (masked vocabularies): top-k then keeps them all
    if (n <= kCand && (!use_k || n >= top_k || tau == -INFINITY)) {
      int n2 = 64;
      while (n2 < n) n2 <<= 1;
      for (int i = n + tid; i < n2; i += blockDim.x) sh.key[i] = 0;      // below every real key
      __syncthreads();
      sort_desc(sh.key, n2);
      for (int i = tid; i < n; i += blockDim.x)
        sh.w[i] = exp((double)key_value(sh.key[i]) * sc.inv_t - m_t);    // exp(-inf) = 0
      __syncthreads();
      if (tid == 0) {
        float t_k = -INFINITY;
        int ns = n;                                     // survivors of top-k: sorted entries 0..ns-1
        double total = Z;
        if (use_k) {
          if (n >= top_k) {
            t_k = key_value(sh.key[top_k - 1]);
            ns = top_k;
            while (ns < n && key_value(sh.key[ns]) == t_k) ++ns;
          }
          total = 0.0;
          for (int i = 0; i < ns; ++i) total += sh.w[i];
        }
        float th = t_k;
        int nk = ns;                                    // kept entries: sorted entries 0..nk-1
        double kept = total;
        bool ok = true;
        if (use_p) {
          ok = false;
          double run = 0.0;
          int i = 0;
          while (i < ns) {
            const float v = key_value(sh.key[i]);
            do { run += sh.w[i]; ++i; } while (i < ns && key_value(sh.key[i]) == v);
            const double frac = run / total;
            if (fabs(frac - (double)top_p) < kNearTie) sh.near_tie = 1;
            if (frac >= (double)top_p) { th = v; nk = i; kept = run; ok = true; break; }
          }
          // top-k survivors always reach P (their own mass is the total); a list
          // without top-k may end before the row's mass does
          if (!ok && use_k) { th = key_value(sh.key[ns - 1]); nk = ns; kept = run; ok = true; }
        } else if (!use_k) {
          kept = 0.0;                                   // no warp at all (short rows): everything is kept
          for (int i = 0; i < n; ++i) kept += sh.w[i];
        }
        while (nk > 0 && sh.w[nk - 1] == 0.0) --nk;     // masses that underflow fp64 are not listed
        sh.theta = th;
        sh.settled = ok ? 1 : 0;
        sh.n_keep = nk;
        sh.z_keep = kept;
      }
      __syncthreads();
      settled = sh.settled != 0;
      theta = sh.theta;
    }
  }
  if (!settled) {
    __syncthreads();
    if (tid == 0) { sh.near_tie = 0; sh.n_keep = -1; }
    theta = general_cutoff<DT>(row, V, lt, top_k, top_p, m, sh);
  }
  if (tid == 0) {
    if (cutoff) cutoff[r] = theta;
    if (flags) flags[r] = sh.near_tie ? SV_FLAG_NEAR_TIE : 0u;
  }
  if (!out.count) return;

  // ---- support of the warped row: token ids ascending, fp64 probabilities ----
  __syncthreads();
  const int nk = sh.n_keep;
  if (nk < 0 || nk > out.cap) {                         // not settled on the list, or too wide
    if (tid == 0) { out.count[r] = -1; out.lse[r] = __builtin_nanf(""); }
    return;
  }
  const double z_keep = sh.z_keep;
  int n2 = 64;
  while (n2 < nk) n2 <<= 1;
  __syncthreads();
  // re-key the kept entries by token id (ascending = descending complement); the position
  // in the value order rides along.  Every slot is rewritten by the thread that read it.
  for (int i = tid; i < n2; i += blockDim.x) {
    uint64_t key = 0;
    if (i < nk) key = ((uint64_t)(0xFFFFFFFFu - key_token(sh.key[i])) << 32) | (uint64_t)i;
    sh.key[i] = key;
  }
  __syncthreads();
  sort_desc(sh.key, n2);
  for (int i = tid; i < nk; i += blockDim.x) {
    const uint64_t key = sh.key[i];
    const size_t at = (size_t)r * out.cap + i;
    out.token[at] = (int32_t)(0xFFFFFFFFu - (uint32_t)(key >> 32));
    out.prob[at] = sh.w[(uint32_t)key] / z_keep;
  }
  if (tid == 0) {
    out.count[r] = nk;
    out.lse[r] = (float)(m_t + log(z_keep));
  }
}

}  // namespace sv

namespace {

int launch_warp(const void* z, int rows, int V, int dtype, float temperature, int top_k, float top_p,
                float* cutoff, uint32_t* flags, const sv::CompactOut& out, sv_stream_t stream) {
  using namespace sv;
  SV_REQUIRE(dtype == SV_F32 || dtype == SV_BF16, SV_ERR_DTYPE);
  SV_REQUIRE(rows >= 0 && V >= 1 && top_p > 0.f, SV_ERR_INVALID_ARG);
  Scale sc;
  SV_REQUIRE(scale_of(temperature, &sc), SV_ERR_INVALID_ARG);
  if (rows == 0) return SV_OK;
  SV_REQUIRE(z, SV_ERR_NULL);
  SV_REQUIRE(is_aligned(z, elem_bytes(dtype)) && is_aligned(cutoff, 4) && is_aligned(flags, 4), SV_ERR_ALIGN);
  hipStream_t st = as_stream(stream);
  if (dtype == SV_F32)
    hipLaunchKernelGGL(warp_cutoffs_kernel<DT_F32>, dim3(rows), dim3(kWarpThreads), 0, st, z, V, sc, top_k, top_p,
                       cutoff, flags, out);
  else
    hipLaunchKernelGGL(warp_cutoffs_kernel<DT_BF16>, dim3(rows), dim3(kWarpThreads), 0, st, z, V, sc, top_k, top_p,
                       cutoff, flags, out);
  return launch_status();
}

}  // namespace

extern "C" int sv_warp_cutoffs(const void* z, int rows, int V, int dtype, float temperature, int top_k,
                               float top_p, float* cutoff, uint32_t* flags_or_null, sv_stream_t stream) {
  SV_REQUIRE(cutoff || rows <= 0, SV_ERR_NULL);
  return launch_warp(z, rows, V, dtype, temperature, top_k, top_p, cutoff, flags_or_null, sv::CompactOut{}, stream);
}

extern "C" int sv_warp_compact(const void* z, int rows, int V, int dtype, float temperature, int top_k,
                               float top_p, int cap, int32_t* count, int32_t* token, double* prob, float* lse,
                               float* cutoff_or_null, uint32_t* flags_or_null, sv_stream_t stream) {
  using namespace sv;
  SV_REQUIRE(cap >= 1 && cap <= SV_SUPPORT_MAX_CAP, SV_ERR_INVALID_ARG);
  SV_REQUIRE((count && token && prob && lse) || rows <= 0, SV_ERR_NULL);
  SV_REQUIRE(is_aligned(count, 4) && is_aligned(token, 4) && is_aligned(prob, 8) && is_aligned(lse, 4),
             SV_ERR_ALIGN);
  return launch_warp(z, rows, V, dtype, temperature, top_k, top_p, cutoff_or_null, flags_or_null,
                     CompactOut{count, token, prob, lse, cap}, stream);
}
