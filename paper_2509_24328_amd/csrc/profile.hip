// Profile construction and information gain (the pass that produces the table
// sv_accept_estimate looks up; Sec. 7.3 "Information Gain from S and A" and the
// appendix definition of the observed probability P(T_i | S, A) in the SV paper).
//
//   sv_quantile_edges      equal-count ("adaptive") bin edges of one axis
//   sv_profile_accumulate  joint histogram of (S-bin, A-bin, X-bin) + per-cell sums of X
//   sv_profile_finalize    cell means with global-mean fill, H(X), H(X|S,A), I(X;S,A)
//
// X = min(1, p_t(x)/p_d(x)) is the acceptance probability of a drafted token
// (sv_accept_ratio).  The paper does not say how X is discretised for H(X);
// here n_x equal bins on [0,1], the top one closed.  These kernels see a few
// thousand samples: they are latency-bound, nothing here streams the vocabulary.
#include "sv_bins.hpp"
#include "sv_device.hpp"
#include "sv_host.hpp"

namespace sv {

constexpr int kQuantMax = 8192;     // samples sorted in one workgroup's LDS
constexpr int kQuantThreads = 1024;

__global__ __launch_bounds__(kQuantThreads) void quantile_edges_kernel(const float* values, int n, int n_bins,
                                                                       float lo, float hi, float* edges) {
  __shared__ float key[kQuantMax];
  __shared__ int n_valid;
  const int tid = threadIdx.x, nt = blockDim.x;
  int npad = 2;
  while (npad < n) npad <<= 1;
  if (tid == 0) n_valid = 0;
  __syncthreads();
  int mine = 0;
  for (int j = tid; j < npad; j += nt) {
    float v = INFINITY;                         // padding and NaNs sort to the end
    if (j < n) {
      const float x = values[j];
      if (!isnan(x)) { v = x; ++mine; }
    }
    key[j] = v;
  }
  if (mine) atomicAdd(&n_valid, mine);
  __syncthreads();
  for (int size = 2; size <= npad; size <<= 1) {          // ascending bitonic sort in LDS
    for (int stride = size >> 1; stride > 0; stride >>= 1) {
      for (int t = tid; t < npad / 2; t += nt) {
        const int a = 2 * t - (t & (stride - 1));
        const int b = a + stride;
        const bool up = (a & size) == 0;
        const float ka = key[a], kb = key[b];
        if (up ? (kb < ka) : (ka < kb)) { key[a] = kb; key[b] = ka; }
      }
      __syncthreads();
    }
  }
  const int m = n_valid;
  for (int j = tid; j <= n_bins; j += nt) {
    float e;
    if (j == 0) e = lo;
    else if (j == n_bins) e = hi;
    else e = (m > 0) ? key[(int)(((long)j * m) / n_bins)] : lo;
    edges[j] = e;
  }
}

// X-bin of a ratio: clip to [0,1] in fp32, multiply by n_x, floor, top closed.
__device__ __forceinline__ int x_bin_of(float xc, int n_x) {
  return min(n_x - 1, (int)floorf(__fmul_rn(xc, (float)n_x)));
}

__global__ void profile_accumulate_kernel(const float* S, const float* A, const float* ratio, int n,
                                          const float* edges_s, int n_s, const float* edges_a, int n_a,
                                          int n_x, uint32_t* counts, double* sum_x) {
  __shared__ float e_lds[kEdgeLds];
  const int j = blockIdx.x * blockDim.x + threadIdx.x;
  float s = 0.f, a = 0.f, r = 0.f;
  if (j < n) { s = S[j]; a = A[j]; r = ratio[j]; }
  const bool in_lds = stage_edges(e_lds, edges_s, n_s, edges_a, n_a);
  if (j >= n || isnan(s) || isnan(a) || isnan(r)) return;
  const float* es = in_lds ? e_lds : edges_s;
  const float* ea = in_lds ? e_lds + n_s + 1 : edges_a;
  const int cell = bin_of(s, es, n_s) * n_a + bin_of(a, ea, n_a);
  const float xc = fminf(1.f, fmaxf(0.f, r));
  atomicAdd(&counts[(size_t)cell * n_x + x_bin_of(xc, n_x)], 1u);
  atomicAdd(&sum_x[cell], (double)xc);
}

constexpr int kFinThreads = 256;
constexpr int kFinMaxX = 1024;

__device__ __forceinline__ double plogp(double c, double tot) {   // -(c/tot) log2(c/tot), 0 for c = 0
  if (!(c > 0.0)) return 0.0;
  const double p = c / tot;
  return -p * log2(p);
}

__global__ __launch_bounds__(kFinThreads) void profile_finalize_kernel(const uint32_t* counts, const double* sum_x,
                                                                       int n_s, int n_a, int n_x, float* table,
                                                                       double* info) {
  __shared__ BlockScratch red;
  __shared__ unsigned long long marg[kFinMaxX];     // marginal counts of the X bins
  const int tid = threadIdx.x, nt = blockDim.x;
  const int cells = n_s * n_a;
  for (int x = tid; x < n_x; x += nt) marg[x] = 0ull;
  __syncthreads();
  // pass 1: totals and X marginals
  double my_n = 0.0, my_sum = 0.0;
  for (int c = tid; c < cells; c += nt) {
    const uint32_t* row = counts + (size_t)c * n_x;
    unsigned long long cn = 0;
    for (int x = 0; x < n_x; ++x) {
      const uint32_t v = row[x];
      cn += v;
      if (v) atomicAdd(&marg[x], (unsigned long long)v);
    }
    my_n += (double)cn;
    my_sum += sum_x[c];
  }
  const double N = block_sum_f64(my_n, red);        // exact: integers below 2^53
  const double total = block_sum_f64(my_sum, red);
  const double glob = N > 0.0 ? total / N : 0.0;
  // pass 2: table and conditional entropy
  double my_h = 0.0;
  for (int c = tid; c < cells; c += nt) {
    const uint32_t* row = counts + (size_t)c * n_x;
    unsigned long long cn = 0;
    for (int x = 0; x < n_x; ++x) cn += row[x];
    if (cn == 0) {
      table[c] = (float)glob;
    } else {
      const double dn = (double)cn;
      table[c] = (float)(sum_x[c] / dn);
      double h = 0.0;
      for (int x = 0; x < n_x; ++x) h += plogp((double)row[x], dn);
      my_h += dn / N * h;
    }
  }
  const double h_cond = block_sum_f64(my_h, red);
  double my_hx = 0.0;
  if (N > 0.0)
    for (int x = tid; x < n_x; x += nt) my_hx += plogp((double)marg[x], N);
  const double h_x = block_sum_f64(my_hx, red);
  if (tid == 0) {
    info[0] = h_x;
    info[1] = h_cond;
    info[2] = h_x - h_cond;
  }
}

}  // namespace sv

extern "C" int sv_quantile_edges(const float* values, int n, int n_bins, float lo, float hi, float* edges,
                                 sv_stream_t stream) {
  using namespace sv;
  SV_REQUIRE(n >= 0 && n_bins >= 1, SV_ERR_INVALID_ARG);
  SV_REQUIRE(n <= kQuantMax, SV_ERR_TOO_LARGE);
  SV_REQUIRE(edges && (values || n == 0), SV_ERR_NULL);
  SV_REQUIRE(is_aligned(values, 4) && is_aligned(edges, 4), SV_ERR_ALIGN);
  hipLaunchKernelGGL(quantile_edges_kernel, dim3(1), dim3(kQuantThreads), 0, as_stream(stream), values, n,
                     n_bins, lo, hi, edges);
  return launch_status();
}

extern "C" int sv_profile_accumulate(const float* S, const float* A, const float* ratio, int n,
                                     const float* edges_s, int n_s, const float* edges_a, int n_a, int n_x,
                                     uint32_t* counts, double* sum_x, sv_stream_t stream) {
  using namespace sv;
  SV_REQUIRE(n >= 0 && n_s >= 1 && n_a >= 1 && n_x >= 1, SV_ERR_INVALID_ARG);
  SV_REQUIRE(n_x <= kFinMaxX, SV_ERR_TOO_LARGE);
  if (n == 0) return SV_OK;
  SV_REQUIRE(S && A && ratio && edges_s && edges_a && counts && sum_x, SV_ERR_NULL);
  SV_REQUIRE(is_aligned(S, 4) && is_aligned(A, 4) && is_aligned(ratio, 4) && is_aligned(edges_s, 4) &&
                 is_aligned(edges_a, 4) && is_aligned(counts, 4) && is_aligned(sum_x, 8),
             SV_ERR_ALIGN);
  const int threads = 256;
  hipLaunchKernelGGL(profile_accumulate_kernel, dim3((n + threads - 1) / threads), dim3(threads), 0,
                     as_stream(stream), S, A, ratio, n, edges_s, n_s, edges_a, n_a, n_x, counts, sum_x);
  return launch_status();
}

extern "C" int sv_profile_finalize(const uint32_t* counts, const double* sum_x, int n_s, int n_a, int n_x,
                                   float* table, double* info, sv_stream_t stream) {
  using namespace sv;
  SV_REQUIRE(n_s >= 1 && n_a >= 1 && n_x >= 1, SV_ERR_INVALID_ARG);
  SV_REQUIRE(n_x <= kFinMaxX && (long long)n_s * n_a <= 0x7fffffffLL, SV_ERR_TOO_LARGE);
  SV_REQUIRE(counts && sum_x && table && info, SV_ERR_NULL);
  SV_REQUIRE(is_aligned(counts, 4) && is_aligned(sum_x, 8) && is_aligned(table, 4) && is_aligned(info, 8),
             SV_ERR_ALIGN);
  hipLaunchKernelGGL(profile_finalize_kernel, dim3(1), dim3(kFinThreads), 0, as_stream(stream), counts, sum_x,
                     n_s, n_a, n_x, table, info);
  return launch_status();
}
