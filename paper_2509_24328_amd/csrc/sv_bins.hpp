// Bin rules of the (S, A) profile grid, shared by the estimate lookup and the
// profile construction kernels (appendix definition of P(T_i | S, A) in the SV
// paper): half-open bins [e_j, e_{j+1}) over ascending edges, the top bin
// closed, values outside clamped, NaN -> bin 0.
#pragma once

#include <hip/hip_runtime.h>

namespace sv {

__device__ __forceinline__ int bin_of(float v, const float* edges, int n) {
  if (isnan(v)) return 0;
  int idx = 0;
  for (int j = 1; j <= n; ++j)
    if (edges[j] <= v) idx = j;
  return min(idx, n - 1);
}

// |v - e_j| <= 1e-5 in fp32 for an interior edge, or v is NaN.
__device__ __forceinline__ bool near_edge(float v, const float* edges, int n) {
  if (isnan(v)) return true;
  for (int j = 1; j < n; ++j)
    if (fabsf(__fsub_rn(v, edges[j])) <= 1e-5f) return true;
  return false;
}

constexpr int kEdgeLds = 1024;    // edges of both axes kept in LDS when they fit

// Stage both edge arrays in LDS (one round of loads).  All threads must call;
// returns false (nothing staged) when they do not fit.
__device__ __forceinline__ bool stage_edges(float* e_lds, const float* edges_s, int n_s,
                                            const float* edges_a, int n_a) {
  if (n_s + n_a + 2 > kEdgeLds) return false;
  for (int t = threadIdx.x; t < n_s + n_a + 2; t += blockDim.x)
    e_lds[t] = (t <= n_s) ? edges_s[t] : edges_a[t - n_s - 1];
  __syncthreads();
  return true;
}

}  // namespace sv
