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
//   select   tau = that bound (top-k); top-p alone has no K: the 48-th largest lane
//            maximum if those 48 already carry P of the row's mass, else the 256-th
//            (a guess of how deep the nucleus reaches)
//   sweep 2  (from cache) append every entry >= tau to a list in LDS
//   settle   sort the list, read off the K-th largest value, walk the groups of equal
//            value until their mass reaches P
// The list is exact whenever it holds at least K entries and (top-p alone) at
// least P of the row's mass; a list that does not settle a top-p row is rebuilt
// once with a lower tau (the 384-th lane maximum).  Otherwise - flat rows, huge K,
// more than 2048 candidates - the general path takes over: radix selection on an
// order-preserving 32-bit key of the logit (11 + 11 + 10 bits; bfloat16 rows are
// resolved after two levels), one histogram sweep of counts and masses per level.
// Masses are fp64 sums of exponentials everywhere: on the candidate path in a fixed
// order (the row total of top-p alone comes from the fp32 sweep), on the general
// path accumulated per bin with LDS fp64 atomics, i.e. in an order that can change
// from run to run in the last bits; a top-p decision within 3e-6 of P is flagged
// SV_FLAG_NEAR_TIE, which covers that by ten orders of magnitude.
//
// sv_warp_compact is the same kernel with one more step: the kept entries of a
// settled list are the whole support of the warped distribution, so their token
// ids (ascending) and fp64 probabilities are written out and everything
// downstream can work on a few dozen entries per row instead of V.
#include "sv_device.hpp"
#include "sv_host.hpp"

// Phase marks: empty in the library; a profiling build may define
// SV_PHASE_MARK(n) to record a clock at the boundaries of the kernel's phases.
#ifndef SV_PHASE_MARK
#define SV_PHASE_MARK(n)
#endif

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
      double mass[kBins];      // fp64: a bin may collect 1e5 nearly equal terms (a flat row at a
                               // high temperature), whose fp32 sum would be off by 1e-4
    };
    struct {                   // candidate path
      uint64_t key[kCand];     // (order key of the value, ~token id): sorted descending
      double w[kCand];         // masses exp((z - m) / T) of the sorted candidates
      uint32_t lane_key[kWarpThreads];   // upper 16 bits of the order key of each lane's maximum
    };
  };
  uint32_t tau_key;
  float theta;
  int n_cand, settled, n_keep, out_done, first_reach, near_any;
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
    const double mm = sh.mass[d];
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
    for (int d = tid; d < kBins; d += blockDim.x) { sh.cnt[d] = 0; sh.mass[d] = 0.0; }
    __syncthreads();
    visit_range<DT, false, 1>(row, nullptr, 0, V, [&](int, float v, float) {   // (one vector at a time: few registers)
      const uint32_t key = okey(v);
      if (under_prefix(key, prefix, level) && v >= floor_v) {
        const uint32_t d = digit_of(key, level);
        atomicAdd(&sh.cnt[d], 1u);
        atomicAdd(&sh.mass[d], (double)exp2_fast(__builtin_fmaf(v, lt, -c_ref)));
      }
    });
    __syncthreads();
  };

  // sweep 2: level 0 over everything
  histogram(0, 0u, -INFINITY);
  double total0 = 0.0;
  {
    double part = 0.0;
    for (int d = tid; d < kBins; d += blockDim.x) part += sh.mass[d];
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
    // level 0 again (the top-k levels have overwritten it; keeping a copy would cost the 16 KB of LDS
    // that decide whether three or four workgroups fit a compute unit, and this path is the rare one):
    // digits above dk0 survive whole, dk0 in part, below not at all
    if (use_k) histogram(0, 0u, -INFINITY);
    for (int d = tid; d < kBins; d += blockDim.x) {
      double mm = sh.mass[d];
      uint32_t c = mm > 0.0 ? 1u : 0u;             // counts only mark non-empty bins here
      if (use_k) {
        if (d < dk0) { mm = 0.0; c = 0u; }
        else if (d == dk0) { mm = surv_in_dk0; c = 1u; }
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

// The four largest tagged keys a lane has seen (k1 >= k2 >= k3 >= k4, unsigned order).
// Key of a 16-byte vector of the row: the upper 16 order-preserving bits of its
// largest entry on top, below them the lane's vector step, from which the lane
// recovers the vector's position.  For fp32 rows the 16 bits order the maxima
// coarsely; that is enough, because the keys only decide which vectors are read
// again and whether a lane may hide one.
struct Top4 {
  uint32_t k1 = 0, k2 = 0, k3 = 0, k4 = 0;
  __device__ __forceinline__ void add(uint32_t key) {
    uint32_t t = key;
    const uint32_t n1 = max(k1, t); t = min(k1, t);
    const uint32_t n2 = max(k2, t); t = min(k2, t);
    const uint32_t n3 = max(k3, t); t = min(k3, t);
    k1 = n1; k2 = n2; k3 = n3; k4 = max(k4, t);
  }
};

constexpr int kTagSteps = 1 << 16;   // vector steps per lane that fit the 16-bit tag

// Sweep 1 for rows made of whole, aligned vectors: the online (max, sum-exp) of
// sweep_online plus the lane's four largest vector maxima with their positions.
template <int DT>
__device__ __forceinline__ void sweep_online_top4(const void* row, int V, Online& acc, Top4& top, const float L) {
  constexpr int EPV = Elem<DT>::per_vec;
  const int tid = threadIdx.x;
  constexpr int nt = kWarpThreads;
  const u32x4* p = reinterpret_cast<const u32x4*>(row);
  const int nvec = V / EPV;
  auto add_vec = [&](const u32x4& q, int i) {
    float f[EPV];
    unpack<DT>(q, f);
    acc.add(f, L);
    float vmax = f[0];
#pragma unroll
    for (int e = 1; e + 1 < EPV; e += 2) vmax = fmaxf(fmaxf(vmax, f[e]), f[e + 1]);
    vmax = fmaxf(vmax, f[EPV - 1]);
    top.add((okey(vmax) & 0xFFFF0000u) | (uint32_t)(i / nt));     // i = tid + step * nt
  };
  int i = tid;
  for (; i + 3 * nt < nvec; i += 4 * nt) {
    const u32x4 q0 = __builtin_nontemporal_load(p + i), q1 = __builtin_nontemporal_load(p + i + nt),
                q2 = __builtin_nontemporal_load(p + i + 2 * nt), q3 = __builtin_nontemporal_load(p + i + 3 * nt);
    add_vec(q0, i); add_vec(q1, i + nt); add_vec(q2, i + 2 * nt); add_vec(q3, i + 3 * nt);
  }
  for (; i < nvec; i += nt) add_vec(__builtin_nontemporal_load(p + i), i);
}

__device__ __forceinline__ uint64_t shfl_u64(uint64_t v, int src) {
  const uint32_t lo = __shfl((uint32_t)v, src, kWave), hi = __shfl((uint32_t)(v >> 32), src, kWave);
  return ((uint64_t)hi << 32) | lo;
}
__device__ __forceinline__ double shfl_f64(double v, int src) {
  int lo = __double2loint(v), hi = __double2hiint(v);
  lo = __shfl(lo, src, kWave);
  hi = __shfl(hi, src, kWave);
  return __hiloint2double(hi, lo);
}

// Descending bitonic sort of one 64-bit key per lane inside a wavefront: the first n2
// lanes (a power of two) are sorted among themselves, which is all that is needed
// when the other lanes hold zeros.
__device__ __forceinline__ uint64_t wave_sort_desc(uint64_t key, int n2 = kWave) {
  const int lane = threadIdx.x & 63;
  for (int k2 = 2; k2 <= n2; k2 <<= 1) {
    for (int j = k2 >> 1; j > 0; j >>= 1) {
      const uint64_t other = shfl_u64(key, lane ^ j);
      const bool desc = (lane & k2) == 0, lower = (lane & j) == 0;
      const uint64_t hi = key > other ? key : other, lo = key > other ? other : key;
      key = (lower == desc) ? hi : lo;
    }
  }
  return key;
}

// Descending sort of keys[0..n), n <= 512 distinct non-zero keys, by a 512-lane
// workgroup: every wavefront sorts 64 keys with shuffles, then every key finds its
// rank by counting the larger keys of the other seven runs (binary searches in
// lock-step, so that their LDS reads overlap).  tmp: n further slots.  keys[n..512)
// end up zero.  Far fewer barriers than a bitonic network in LDS.
__device__ __forceinline__ void sort_desc_runs(uint64_t* keys, uint64_t* tmp, int n) {
  constexpr int kRuns = kWarpThreads / kWave;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  uint64_t key = tid < n ? keys[tid] : 0;
  key = wave_sort_desc(key);
  __syncthreads();                                     // all keys read before any is overwritten
  keys[tid] = key;
  __syncthreads();
  int pos[kRuns];
#pragma unroll
  for (int r = 0; r < kRuns; ++r) pos[r] = 0;
  for (int step = kWave; step > 0; step >>= 1) {
#pragma unroll
    for (int r = 0; r < kRuns; ++r) {
      const int probe = pos[r] + step;
      if (r != wave && probe <= kWave && keys[r * kWave + probe - 1] > key) pos[r] = probe;
    }
  }
  int rank = lane;
#pragma unroll
  for (int r = 0; r < kRuns; ++r) rank += (r != wave) ? pos[r] : 0;
  if (key != 0) tmp[rank] = key;
  __syncthreads();
  keys[tid] = tid < n ? tmp[tid] : 0;
  __syncthreads();
}


// top-p alone has no K and guesses the depth of the nucleus from the lane maxima: a
// list of about rank + rank^2 / 1024 entries, short enough for the one-wavefront
// settle when the largest 48 lane maxima already carry P of the row's mass, a deeper
// one otherwise
constexpr int kNucleusRank = 48;
constexpr int kNucleusRank2 = 256;

// One row (r of tensor z) by the whole workgroup.
template <int DT>
__device__ __forceinline__ void warp_row(const void* z, const int r, int V, const Scale sc, int top_k, float top_p,
                                         float* cutoff, uint32_t* flags, const CompactOut out, WarpShared& sh) {
  const int tid = threadIdx.x;
  const void* row = static_cast<const char*>(z) + (size_t)r * V * Elem<DT>::bytes;
  const float lt = sc.L;

  // sweep 1: maximum, normaliser, bad-row detection (NaN poisons the sum, +inf the maximum)
  SV_PHASE_MARK(0)
  Online acc[1];
  acc[0].init();
  Top4 top;
  const bool tagged = aligned16(row) && V % Elem<DT>::per_vec == 0 &&
                      V / Elem<DT>::per_vec <= kTagSteps * kWarpThreads;
  if (tagged) sweep_online_top4<DT>(row, V, acc[0], top, lt);
  else sweep_online<DT, false, false>(row, V, 0, 1, acc[0], lt);
  MS merged[1];
  block_merge<1>(acc, sh.mg, merged, lt);
  const float m = merged[0].m;
  SV_PHASE_MARK(1)
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

  // The rank-th largest of the 512 lane maxima, to the 16 upper bits of its order key
  // (exact for bfloat16, rounded down for fp32): a lower bound of the rank-th largest
  // entry of the row.  Wavefront 0 holds eight maxima per lane and bisects the 16 bits
  // with ballots.
  sh.lane_key[tid] = okey(acc[0].m) >> 16;
  __syncthreads();
  auto lane_max_of_rank = [&](int rank) {
    if (tid < kWave) {
      uint32_t kk[kWarpThreads / kWave];
#pragma unroll
      for (int j = 0; j < kWarpThreads / kWave; ++j) kk[j] = sh.lane_key[tid + kWave * j];
      uint32_t t = 0;
      for (int bit = 15; bit >= 0; --bit) {
        const uint32_t cand = t | (1u << bit);
        int c = 0;
#pragma unroll
        for (int j = 0; j < kWarpThreads / kWave; ++j) c += __popcll(__ballot(kk[j] >= cand));
        if (c >= rank) t = cand;
      }
      if (tid == 0) sh.tau_key = t << 16;
    }
    __syncthreads();
    const uint32_t tk = sh.tau_key;
    // keys at or below that of -inf (lanes without a finite entry) mean: no bound
    return tk <= (okey(-INFINITY) & 0xFFFF0000u) ? -INFINITY : from_okey(tk);
  };

  // The same decisions for a list of at most 64 entries, taken by wavefront 0 alone
  // with shuffles (no barriers, no serial walk); it also writes the row's support.
  auto settle_wave = [&](int n) {
    const int lane = tid;                                // wavefront 0: tid = lane
    uint64_t key = lane < n ? sh.key[lane] : 0;
    int n2 = 2;
    while (n2 < n) n2 <<= 1;
    key = wave_sort_desc(key, n2);
    const bool valid = lane < n;
    const float v = valid ? key_value(key) : -INFINITY;
    const double w = valid ? exp((double)v * sc.inv_t - m_t) : 0.0;
    float t_k = -INFINITY;
    int ns = n;
    double total = Z;
    if (use_k) {
      if (n >= top_k) {
        t_k = __shfl(v, top_k - 1, kWave);
        ns = __popcll(__ballot(valid && v >= t_k));      // a prefix: the list is sorted
      }
      total = wave_sum_f64(lane < ns ? w : 0.0);
    }
    float th = t_k;
    int nk = ns;
    double kept = total;
    bool ok = true;
    int near = 0;
    if (use_p) {
      double incl = lane < ns ? w : 0.0;                 // inclusive prefix masses
#pragma unroll
      for (int off = 1; off < kWave; off <<= 1) {
        const double o = shfl_f64(incl, max(lane - off, 0));
        if (lane >= off) incl += o;
      }
      const float v_next = __shfl(v, min(lane + 1, kWave - 1), kWave);
      const bool group_end = lane < ns && (lane == ns - 1 || v_next != v);
      const double frac = incl / total;
      const unsigned long long reach = __ballot(group_end && frac >= (double)top_p);
      int d = reach ? (int)__builtin_ctzll(reach) : -1;
      if (d < 0 && use_k) d = ns - 1;                    // survivors of top-k are their own total
      ok = d >= 0;
      if (ok) {
        near = __ballot(group_end && lane <= d && fabs(frac - (double)top_p) < kNearTie) != 0;
        th = __shfl(v, d, kWave);
        nk = d + 1;
        kept = shfl_f64(incl, d);
      }
    } else if (!use_k) {
      kept = wave_sum_f64(w);                            // no warp at all (short rows)
    }
    nk = __popcll(__ballot(lane < nk && w > 0.0));       // masses that underflow fp64 are not listed
    if (ok && out.count) {
      if (nk <= out.cap) {
        // order the kept entries by token id and write them out
        uint64_t k2 = lane < nk ? (((uint64_t)(0xFFFFFFFFu - key_token(key)) << 32) | (uint64_t)lane) : 0;
        int m2 = 2;
        while (m2 < nk) m2 <<= 1;
        k2 = wave_sort_desc(k2, m2);
        const double wj = shfl_f64(w, (int)(uint32_t)k2 & 63);
        if (lane < nk) {
          const size_t at = (size_t)r * out.cap + lane;
          out.token[at] = (int32_t)(0xFFFFFFFFu - (uint32_t)(k2 >> 32));
          out.prob[at] = wj / kept;
        }
      }
      if (lane == 0) {
        out.count[r] = nk <= out.cap ? nk : -1;
        out.lse[r] = nk <= out.cap ? (float)(m_t + log(kept)) : __builtin_nanf("");
      }
    }
    if (lane == 0) {
      sh.theta = th;
      sh.settled = ok ? 1 : 0;
      sh.n_keep = ok ? nk : -1;
      sh.z_keep = kept;
      sh.near_tie = ok ? near : 0;
      sh.out_done = ok ? 1 : 0;
    }
  };

  // Settle top-k / top-p on the list sh.key[0 .. sh.n_cand) of all entries >= tau.
  // Called by all threads; true when the list decides the row (then sh.theta,
  // sh.n_keep, sh.z_keep are set and the kept entries are sh.key[0 .. n_keep)).
  auto settle = [&](float tau) {
    const int n = sh.n_cand;
    if (n <= kWave && (!use_k || n >= top_k || tau == -INFINITY)) {
      if (tid < kWave) settle_wave(n);
      __syncthreads();
      return sh.settled != 0;
    }
    // fewer than K candidates happens only when tau = -inf lists every finite entry
    // of the row (masked vocabularies): top-k then keeps them all
    if (!(n <= kCand && (!use_k || n >= top_k || tau == -INFINITY))) return false;
    if (n <= kWarpThreads) {
      sort_desc_runs(sh.key, reinterpret_cast<uint64_t*>(sh.w), n);    // (the masses are not there yet)
    } else {
      int n2 = kWarpThreads;
      while (n2 < n) n2 <<= 1;
      for (int i = n + tid; i < n2; i += blockDim.x) sh.key[i] = 0;    // below every real key
      __syncthreads();
      sort_desc(sh.key, n2);
    }
    SV_PHASE_MARK(4)
    for (int i = tid; i < n; i += blockDim.x)
      sh.w[i] = exp((double)key_value(sh.key[i]) * sc.inv_t - m_t);
    __syncthreads();
    SV_PHASE_MARK(5)
    // Every lane owns a run of consecutive sorted entries; the masses of the
    // survivors are prefix-summed over the workgroup (fp64), then every lane looks
    // at the ends of groups of equal value inside its run.
    float t_k = -INFINITY;
    int ns = n;                                       // survivors of top-k: sorted entries 0..ns-1
    if (use_k && n >= top_k) {
      t_k = key_value(sh.key[top_k - 1]);
      int lo = top_k, hi = n;                         // first entry below t_k
      while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (key_value(sh.key[mid]) >= t_k) lo = mid + 1; else hi = mid;
      }
      ns = lo;
    }
    constexpr int kRun = kCand / kWarpThreads;
    const int i0 = tid * kRun;
    double wv[kRun];
    float vv[kRun + 1];
    double mine = 0.0;
#pragma unroll
    for (int j = 0; j < kRun; ++j) {
      const int i = i0 + j;
      wv[j] = i < ns ? sh.w[i] : 0.0;
      vv[j] = i < n ? key_value(sh.key[i]) : -INFINITY;
      mine += wv[j];
    }
    vv[kRun] = i0 + kRun < n ? key_value(sh.key[i0 + kRun]) : -INFINITY;
    double incl = mine;                               // inclusive scan of the lanes' sums
    const int lane = tid & 63, wave = tid >> 6;
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
      const double o = shfl_f64(incl, max(lane - off, 0));
      if (lane >= off) incl += o;
    }
    if (lane == kWave - 1) sh.red.d[wave] = incl;
    if (tid == 0) { sh.first_reach = 0x7fffffff; sh.near_any = 0; }
    __syncthreads();
    double base = incl - mine, surv_total = 0.0;
    for (int w = 0; w < (int)(blockDim.x >> 6); ++w) {
      const double tw = sh.red.d[w];
      if (w < wave) base += tw;
      surv_total += tw;
    }
    const double total = use_k ? surv_total : Z;
    double run[kRun], fr[kRun];
    bool gend[kRun];
    {
      double acc = base;
#pragma unroll
      for (int j = 0; j < kRun; ++j) {
        const int i = i0 + j;
        acc += wv[j];
        run[j] = acc;
        fr[j] = acc / total;
        gend[j] = i < ns && (i == ns - 1 || vv[j + 1] != vv[j]);
        if (use_p && gend[j] && fr[j] >= (double)top_p) atomicMin(&sh.first_reach, i);
      }
    }
    __syncthreads();
    int d = sh.first_reach;
    bool ok = true;
    if (use_p) {
      // top-k survivors always reach P (their own mass is the total); a list
      // without top-k may end before the row's mass does
      if (d == 0x7fffffff) { d = ns - 1; ok = use_k; }
    } else {
      d = ns - 1;                                     // nothing to walk: all survivors are kept
    }
    if (ok) {
#pragma unroll
      for (int j = 0; j < kRun; ++j) {
        const int i = i0 + j;
        if (use_p && gend[j] && i <= d && fabs(fr[j] - (double)top_p) < kNearTie) atomicOr(&sh.near_any, 1);
        if (i == d) {
          sh.theta = use_p ? vv[j] : t_k;
          sh.z_keep = run[j];
        }
      }
    }
    __syncthreads();
    if (tid == 0) {
      int nk = d + 1;
      while (ok && nk > 0 && sh.w[nk - 1] == 0.0) --nk;   // masses that underflow fp64 are not listed
      sh.settled = ok ? 1 : 0;
      sh.n_keep = ok ? nk : -1;
      sh.near_tie = ok ? sh.near_any : 0;
    }
    __syncthreads();
    return sh.settled != 0;
  };

  bool settled = false;
  if (tid == 0) { sh.n_cand = 0; sh.near_tie = 0; sh.settled = 0; sh.n_keep = -1; sh.out_done = 0; }
  __syncthreads();

  // ---- attempt 1 (tagged rows): only the lanes' largest vectors are read again.
  // A lane whose fourth-largest vector may reach tau may hide a fifth one that
  // does: such a lane (rare) walks all of its vectors again instead.
  if (tagged && V > kCand && (!use_k || top_k <= kWarpThreads)) {
    float tau = lane_max_of_rank(use_k ? top_k : kNucleusRank);
    if (!use_k) {
      // top-p alone: does the mass of the lane maxima above tau already reach P?  Then the
      // list above tau certainly does; otherwise ask for a deeper list straight away.
      if (tid < kWave) {
        const uint32_t t16 = sh.tau_key >> 16;
        double above = 0.0;
#pragma unroll
        for (int j = 0; j < kWarpThreads / kWave; ++j) {
          const uint32_t k16 = sh.lane_key[tid + kWave * j];
          // (the 16-bit key rounds an fp32 maximum down: the sum is a lower bound)
          if (k16 >= t16 && k16 > (okey(-INFINITY) >> 16)) above += exp((double)from_okey(k16 << 16) * sc.inv_t - m_t);
        }
        above = wave_sum_f64(above);
        if (tid == 0) sh.z_keep = above;
      }
      __syncthreads();
      const bool deep = sh.z_keep < (double)top_p * Z * (1.0 + 1e-6);
      __syncthreads();
      if (deep) tau = lane_max_of_rank(kNucleusRank2);
    }
    SV_PHASE_MARK(2)
    const uint32_t tau_key = sh.tau_key;
    if (tau > -INFINITY) {
      constexpr int EPV = Elem<DT>::per_vec;
      const u32x4* p = reinterpret_cast<const u32x4*>(row);
      auto list_vector = [&](uint32_t vec) {
        float f[EPV];
        unpack<DT>(p[vec], f);
#pragma unroll
        for (int e = 0; e < EPV; ++e) {
          if (f[e] >= tau && f[e] > -INFINITY) {
            const int at = atomicAdd(&sh.n_cand, 1);
            if (at < kCand)
              sh.key[at] = ((uint64_t)okey(f[e]) << 32) | (uint64_t)(0xFFFFFFFFu - (vec * EPV + (uint32_t)e));
          }
        }
      };
      if (top.k4 >= tau_key) {
        for (uint32_t vec = (uint32_t)tid; vec < (uint32_t)(V / EPV); vec += kWarpThreads) list_vector(vec);
      } else {
        const uint32_t keys[3] = {top.k1, top.k2, top.k3};
#pragma unroll
        for (int q = 0; q < 3; ++q)
          if (keys[q] >= tau_key) list_vector((keys[q] & 0xFFFFu) * kWarpThreads + (uint32_t)tid);
      }
      __syncthreads();
      SV_PHASE_MARK(3)
      settled = settle(tau);
      SV_PHASE_MARK(6)
    }
  }

  // ---- attempt 2: a second sweep (from cache) lists every entry >= tau -------
  if (!settled && (V <= kCand || !use_k || top_k <= kWarpThreads)) {
    float tau = -INFINITY;                              // V <= kCand: every entry is a candidate
    if (V > kCand) tau = lane_max_of_rank(use_k ? top_k : kGuessRank);
    __syncthreads();
    if (tid == 0) sh.n_cand = 0;
    __syncthreads();
    visit_range<DT, false, 4>(row, nullptr, 0, V, [&](int v, float zv, float) {
      if (zv >= tau && zv > -INFINITY) {                // entries at -inf carry no mass and are never listed
        const int at = atomicAdd(&sh.n_cand, 1);        // a few per row: the shared counter is not a bottleneck
        if (at < kCand) sh.key[at] = ((uint64_t)okey(zv) << 32) | (uint64_t)(0xFFFFFFFFu - (uint32_t)v);
      }
    });
    __syncthreads();
    settled = settle(tau);
  }
  float theta = sh.theta;
  if (!settled) {
    __syncthreads();
    if (tid == 0) { sh.near_tie = 0; sh.n_keep = -1; }
    theta = general_cutoff<DT>(row, V, lt, top_k, top_p, m, sh);
  }
  if (tid == 0) {
    if (cutoff) cutoff[r] = theta;
    if (flags) flags[r] = sh.near_tie ? SV_FLAG_NEAR_TIE : 0u;
  }
  if (!out.count || (settled && sh.out_done)) return;    // (the wavefront path has written the support already)

  // ---- support of the warped row: token ids ascending, fp64 probabilities ----
  __syncthreads();
  const int nk = sh.n_keep;
  if (nk < 0 || nk > out.cap) {                         // not settled on the list, or too wide
    if (tid == 0) { out.count[r] = -1; out.lse[r] = __builtin_nanf(""); }
    return;
  }
  const double z_keep = sh.z_keep;
  __syncthreads();
  // re-key the kept entries by token id (ascending = descending complement); the position
  // in the value order rides along.  Every slot is rewritten by the thread that read it.
  int n2 = kWarpThreads;
  while (n2 < nk) n2 <<= 1;
  for (int i = tid; i < n2; i += blockDim.x) {
    uint64_t key = 0;
    if (i < nk) key = ((uint64_t)(0xFFFFFFFFu - key_token(sh.key[i])) << 32) | (uint64_t)i;
    sh.key[i] = key;
  }
  __syncthreads();
  if (nk <= kWarpThreads) sort_desc_runs(sh.key, sh.key + kCand / 2, nk);   // (the list beyond nk is dead)
  else sort_desc(sh.key, n2);
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
  SV_PHASE_MARK(7)
}

// Up to kWarpMaxTensors logit tensors of one vocabulary size in one launch (one workgroup
// per row of any of them): a launch with about two rows per compute unit has nothing to
// put behind the decisions of its last rows and thins out over its final third; more
// rows per launch overlap the decisions of some rows with the sweeps of others.
constexpr int kWarpMaxTensors = SV_WARP_MAX_TENSORS;
struct WarpBatch {
  int n;
  int row_end[kWarpMaxTensors];          // running totals of the tensors' rows
  const void* z[kWarpMaxTensors];
  Scale sc[kWarpMaxTensors];
  int top_k[kWarpMaxTensors];
  float top_p[kWarpMaxTensors];
  float* cutoff[kWarpMaxTensors];
  uint32_t* flags[kWarpMaxTensors];
  CompactOut out[kWarpMaxTensors];
};

// (8 wavefronts per SIMD = four workgroups per compute unit: the decisions of some rows overlap the
// sweeps of others; needs <= 64 VGPRs and <= 40 KB of LDS)
template <int DT>
__global__ __launch_bounds__(kWarpThreads, 8) void warp_cutoffs_kernel(int V, WarpBatch b) {
  __shared__ WarpShared sh;
  int t = 0;
  while (t + 1 < b.n && (int)blockIdx.x >= b.row_end[t]) ++t;
  const int r = (int)blockIdx.x - (t ? b.row_end[t - 1] : 0);
  warp_row<DT>(b.z[t], r, V, b.sc[t], b.top_k[t], b.top_p[t], b.cutoff[t], b.flags[t], b.out[t], sh);
}

}  // namespace sv

namespace {

// Checks and launch of one or several tensors (arrays of length n on the host).
int launch_warp(int n, const void* const* z, const int* rows, int V, int dtype, const float* temperature,
                const int* top_k, const float* top_p, float* const* cutoff, uint32_t* const* flags,
                const sv::CompactOut* outs, bool need_cutoff, sv_stream_t stream) {
  using namespace sv;
  SV_REQUIRE(dtype == SV_F32 || dtype == SV_BF16, SV_ERR_DTYPE);
  SV_REQUIRE(n >= 1 && n <= kWarpMaxTensors && V >= 1, SV_ERR_INVALID_ARG);
  WarpBatch b = {};
  long long total = 0;
  for (int t = 0; t < n; ++t) {
    SV_REQUIRE(rows[t] >= 0 && top_p[t] > 0.f, SV_ERR_INVALID_ARG);
    SV_REQUIRE(scale_of(temperature[t], &b.sc[t]), SV_ERR_INVALID_ARG);
    if (rows[t] > 0) {
      SV_REQUIRE(z[t] && (!need_cutoff || cutoff[t]), SV_ERR_NULL);
      if (outs) SV_REQUIRE(outs[t].count && outs[t].token && outs[t].prob && outs[t].lse, SV_ERR_NULL);
    }
    SV_REQUIRE(is_aligned(z[t], elem_bytes(dtype)) && is_aligned(cutoff ? cutoff[t] : nullptr, 4) &&
                   is_aligned(flags ? flags[t] : nullptr, 4),
               SV_ERR_ALIGN);
    if (outs) {
      SV_REQUIRE(outs[t].cap >= 1 && outs[t].cap <= SV_SUPPORT_MAX_CAP, SV_ERR_INVALID_ARG);
      SV_REQUIRE(is_aligned(outs[t].count, 4) && is_aligned(outs[t].token, 4) && is_aligned(outs[t].prob, 8) &&
                     is_aligned(outs[t].lse, 4),
                 SV_ERR_ALIGN);
      b.out[t] = outs[t];
    }
    total += rows[t];
    SV_REQUIRE(total <= 0x7fffffffLL, SV_ERR_TOO_LARGE);
    b.row_end[t] = (int)total;
    b.z[t] = z[t];
    b.top_k[t] = top_k[t];
    b.top_p[t] = top_p[t];
    b.cutoff[t] = cutoff ? cutoff[t] : nullptr;
    b.flags[t] = flags ? flags[t] : nullptr;
  }
  b.n = n;
  if (total == 0) return SV_OK;
  hipStream_t st = as_stream(stream);
  if (dtype == SV_F32)
    hipLaunchKernelGGL(warp_cutoffs_kernel<DT_F32>, dim3((unsigned)total), dim3(kWarpThreads), 0, st, V, b);
  else
    hipLaunchKernelGGL(warp_cutoffs_kernel<DT_BF16>, dim3((unsigned)total), dim3(kWarpThreads), 0, st, V, b);
  return launch_status();
}

}  // namespace

extern "C" int sv_warp_cutoffs(const void* z, int rows, int V, int dtype, float temperature, int top_k,
                               float top_p, float* cutoff, uint32_t* flags_or_null, sv_stream_t stream) {
  return launch_warp(1, &z, &rows, V, dtype, &temperature, &top_k, &top_p, &cutoff, &flags_or_null, nullptr, true,
                     stream);
}

extern "C" int sv_warp_cutoffs_multi(int n, const void* const* z, const int* rows, int V, int dtype,
                                     const float* temperature, const int* top_k, const float* top_p,
                                     float* const* cutoff, uint32_t* const* flags_or_null, sv_stream_t stream) {
  SV_REQUIRE(n >= 1 && n <= SV_WARP_MAX_TENSORS, SV_ERR_INVALID_ARG);
  SV_REQUIRE(z && rows && temperature && top_k && top_p && cutoff, SV_ERR_NULL);
  return launch_warp(n, z, rows, V, dtype, temperature, top_k, top_p, cutoff, flags_or_null, nullptr, true, stream);
}

extern "C" int sv_warp_compact(const void* z, int rows, int V, int dtype, float temperature, int top_k,
                               float top_p, int cap, int32_t* count, int32_t* token, double* prob, float* lse,
                               float* cutoff_or_null, uint32_t* flags_or_null, sv_stream_t stream) {
  using namespace sv;
  SV_REQUIRE(cap >= 1 && cap <= SV_SUPPORT_MAX_CAP, SV_ERR_INVALID_ARG);
  const CompactOut out{count, token, prob, lse, cap};
  return launch_warp(1, &z, &rows, V, dtype, &temperature, &top_k, &top_p, &cutoff_or_null, &flags_or_null, &out,
                     false, stream);
}

extern "C" int sv_warp_compact_multi(int n, const void* const* z, const int* rows, int V, int dtype,
                                     const float* temperature, const int* top_k, const float* top_p, int cap,
                                     int32_t* const* count, int32_t* const* token, double* const* prob,
                                     float* const* lse, float* const* cutoff_or_null,
                                     uint32_t* const* flags_or_null, sv_stream_t stream) {
  using namespace sv;
  SV_REQUIRE(n >= 1 && n <= SV_WARP_MAX_TENSORS, SV_ERR_INVALID_ARG);
  SV_REQUIRE(z && rows && temperature && top_k && top_p && count && token && prob && lse, SV_ERR_NULL);
  CompactOut outs[SV_WARP_MAX_TENSORS];
  for (int t = 0; t < n; ++t) outs[t] = CompactOut{count[t], token[t], prob[t], lse[t], cap};
  return launch_warp(n, z, rows, V, dtype, temperature, top_k, top_p, cutoff_or_null, flags_or_null, outs, false,
                     stream);
}
