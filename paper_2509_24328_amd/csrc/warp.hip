// sv_warp_cutoffs: per-row cutoff of the sampling warps temperature -> top-k ->
// top-p (the sampling hyper-parameters of the SV paper's appendix table), so
// that the warped distribution is soft-max(z / T) restricted to {v : z_v >= cutoff}.
// Entries of equal value are kept or dropped together.
//
// One workgroup per row, radix selection on an order-preserving 32-bit key of
// the logit (11 + 11 + 10 bits; bfloat16 rows are resolved after two levels
// because their low 16 bits are constant):
//   sweep 1  row maximum (and NaN / +inf detection)
//   sweep 2  level-0 histograms of all entries: count and mass 2^((z-m) L/T)
//   top-k    descend with count histograms of the entries under the current
//            prefix (one sweep per further level); masses ride along
//   top-p    over the survivors of top-k: level 0 comes from the saved level-0
//            masses, further levels need one sweep each
// Masses are summed with LDS float atomics (order not fixed, ~1e-7 relative):
// a top-p decision within 1e-6 of P is flagged SV_FLAG_NEAR_TIE.
#include "sv_device.hpp"
#include "sv_host.hpp"

namespace sv {

constexpr int kWarpThreads = 512;
constexpr int kBins = 2048;

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

struct WarpShared {
  BlockScratch red;
  uint32_t cnt[kBins];
  float mass[kBins];
  float mass0[kBins];        // level-0 masses, kept for the top-p pass
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
      if (fabs(fr - want) < 1e-6) sh.near_tie = 1;
    }
    if (hit || d == 0) { found = d; sh.sel_mass_bin = mm; break; }
    c_above += c;
    m_above += mm;
  }
  sh.sel_digit = found;
  sh.sel_count_above = c_above;
  sh.sel_mass_above = m_above;
}

template <int DT>
__global__ __launch_bounds__(kWarpThreads) void warp_cutoffs_kernel(const void* z, int V, float lt, int top_k,
                                                                    float top_p, float* cutoff, uint32_t* flags) {
  __shared__ WarpShared sh;
  const int tid = threadIdx.x;
  const void* row = static_cast<const char*>(z) + (size_t)blockIdx.x * V * Elem<DT>::bytes;
  constexpr int kLevels = (DT == DT_BF16) ? 2 : 3;

  // sweep 1: maximum, bad-row detection
  float mx = -INFINITY;
  int bad = 0;
  visit_range<DT, false, 4>(row, nullptr, 0, V, [&](int, float v, float) {
    mx = fmaxf(mx, v);
    bad |= (isnan(v) || v == INFINITY) ? 1 : 0;
  });
  mx = wave_max_f32(mx);
  if ((tid & 63) == 0) sh.red.f[tid >> 6] = mx;
  const int any_bad = __syncthreads_or(bad);
  float m = sh.red.f[0];
  for (int w = 1; w < (int)(blockDim.x >> 6); ++w) m = fmaxf(m, sh.red.f[w]);
  __syncthreads();
  if (any_bad || m == -INFINITY) {
    if (tid == 0) { cutoff[blockIdx.x] = __builtin_nanf(""); if (flags) flags[blockIdx.x] = SV_FLAG_BAD_ROW; }
    return;
  }
  const bool use_k = top_k > 0 && top_k < V, use_p = top_p < 1.0f;
  if (!use_k && !use_p) {
    if (tid == 0) { cutoff[blockIdx.x] = -INFINITY; if (flags) flags[blockIdx.x] = 0; }
    return;
  }
  const float c_ref = m * lt;
  if (tid == 0) sh.near_tie = 0;

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
  if (tid == 0) {
    cutoff[blockIdx.x] = theta;
    if (flags) flags[blockIdx.x] = sh.near_tie ? SV_FLAG_NEAR_TIE : 0u;
  }
}

}  // namespace sv

extern "C" int sv_warp_cutoffs(const void* z, int rows, int V, int dtype, float temperature, int top_k,
                               float top_p, float* cutoff, uint32_t* flags_or_null, sv_stream_t stream) {
  using namespace sv;
  SV_REQUIRE(dtype == SV_F32 || dtype == SV_BF16, SV_ERR_DTYPE);
  SV_REQUIRE(rows >= 0 && V >= 1 && temperature > 0.f && top_p > 0.f, SV_ERR_INVALID_ARG);
  if (rows == 0) return SV_OK;
  SV_REQUIRE(z && cutoff, SV_ERR_NULL);
  SV_REQUIRE(is_aligned(z, elem_bytes(dtype)) && is_aligned(cutoff, 4) && is_aligned(flags_or_null, 4),
             SV_ERR_ALIGN);
  const float lt = (float)(1.4426950408889634 / (double)temperature);
  hipStream_t st = as_stream(stream);
  if (dtype == SV_F32)
    hipLaunchKernelGGL(warp_cutoffs_kernel<DT_F32>, dim3(rows), dim3(kWarpThreads), 0, st, z, V, lt, top_k, top_p,
                       cutoff, flags_or_null);
  else
    hipLaunchKernelGGL(warp_cutoffs_kernel<DT_BF16>, dim3(rows), dim3(kWarpThreads), 0, st, z, V, lt, top_k, top_p,
                       cutoff, flags_or_null);
  return launch_status();
}
