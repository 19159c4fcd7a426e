// sv_accept_estimate: lookup of the binned acceptance estimate P^(T_i | S, A)
// (appendix definition of the observed probability in the SV paper).
// One lane per (sequence, position); the profile table and its edges are a few
// hundred floats and stay in cache.  Launch-latency bound.
#include "sv_bins.hpp"
#include "sv_device.hpp"
#include "sv_host.hpp"

namespace sv {

__global__ void accept_estimate_kernel(const float* S, const float* A, int n,
                                       const float* edges_s, int n_s,
                                       const float* edges_a, int n_a,
                                       const float* table, float* p_hat, uint8_t* edge_flag) {
  // the edge arrays are walked by every lane: fetch them once, in one round of
  // loads together with S and A, instead of one dependent load per edge
  __shared__ float e_lds[kEdgeLds];
  const int j = blockIdx.x * blockDim.x + threadIdx.x;
  float s = 0.f, a = 0.f;
  if (j < n) { s = S[j]; a = A[j]; }
  const bool in_lds = stage_edges(e_lds, edges_s, n_s, edges_a, n_a);
  if (j >= n) return;
  const float* es = in_lds ? e_lds : edges_s;
  const float* ea = in_lds ? e_lds + n_s + 1 : edges_a;
  p_hat[j] = table[bin_of(s, es, n_s) * n_a + bin_of(a, ea, n_a)];
  if (edge_flag) edge_flag[j] = (near_edge(s, es, n_s) || near_edge(a, ea, n_a)) ? 1 : 0;
}

}  // namespace sv

extern "C" int sv_accept_estimate(const float* S, const float* A, int n,
                                  const float* edges_s, int n_s, const float* edges_a, int n_a,
                                  const float* table, float* p_hat, uint8_t* edge_flag_or_null,
                                  sv_stream_t stream) {
  using namespace sv;
  SV_REQUIRE(n >= 0 && n_s >= 1 && n_a >= 1, SV_ERR_INVALID_ARG);
  if (n == 0) return SV_OK;
  SV_REQUIRE(S && A && edges_s && edges_a && table && p_hat, SV_ERR_NULL);
  SV_REQUIRE(is_aligned(S, 4) && is_aligned(A, 4) && is_aligned(edges_s, 4) && is_aligned(edges_a, 4) &&
                 is_aligned(table, 4) && is_aligned(p_hat, 4),
             SV_ERR_ALIGN);
  const int threads = 256;
  TapScope tap(SV_KERNEL_ACCEPT_ESTIMATE, as_stream(stream));
  hipLaunchKernelGGL(accept_estimate_kernel, dim3((n + threads - 1) / threads), dim3(threads), 0,
                     as_stream(stream), S, A, n, edges_s, n_s, edges_a, n_a, table, p_hat,
                     edge_flag_or_null);
  return launch_status();
}
