// sv_select_length: verification length per sequence from the acceptance
// estimates (Sec. 5 of the SV paper: P_gamma(N), E(N | gamma), estimated
// goodput, incremental search, batch-level greedy rule).
//
// With c[b,j] = prod_{i<=j} p_hat[b,i] the expected accepted length of
// verifying gamma tokens of sequence b is sum_{j<gamma} c[b,j], so the token
// whose verification raises the expected accepted length most (the choice of
// the batch-level greedy rule, Sec. 5, batch scheduling) is always the
// largest not-yet-taken c.  Because c is non-increasing along a sequence,
// sorting all (b,j) by (c descending, b, j ascending) reproduces the greedy
// order.  One workgroup: products (one lane per sequence); pairwise merging of
// the per-sequence lists in LDS (they are sorted already); the running sum E_M
// is defined in exactly that order (fp64, one addition after another, so that
// the integer outputs do not depend on a reduction tree) - a parallel scan with
// an error bound decides every comparison that is not a near tie, one lane
// re-sums in order otherwise; goodput and first-peak search in parallel; counts
// and offsets.  Launch-latency bound at the paper's batch sizes (12 us at 512
// keys; 55 us at 4096, 120 us at 8192).
#include "sv_bins.hpp"
#include "sv_device.hpp"
#include "sv_host.hpp"

// Phase marks: empty in the library; a profiling build may define
// SV_PHASE_MARK(n) to record a clock at the boundaries of the kernel's phases.
#ifndef SV_PHASE_MARK
#define SV_PHASE_MARK(n)
#endif

namespace sv {

constexpr int kSelThreads = 1024;
constexpr int kSelMax = SV_SELECT_MAX_KEYS;   // power of two
constexpr int kMergeMax = kSelMax / 2;         // up to here the upper half of the key arrays is a second buffer

__device__ __forceinline__ double clean_p(float p) {
  if (isnan(p)) return 0.0;
  return fmin(fmax((double)p, 0.0), 1.0);
}

// Exclusive scan of cnt[b] + 1 over b = 0..B-1 by the whole workgroup; writes
// gamma[b] = cnt[b] and t_offsets[0..B].  cnt may live in LDS or global memory;
// `part` holds one int of LDS per wavefront.  Integer sums: exact in any order.
__device__ __forceinline__ void offsets_scan(const int* cnt, int B, int32_t* gamma, int32_t* t_offsets,
                                             int* part) {
  const int tid = threadIdx.x, nt = blockDim.x;
  const int lane = tid & (kWave - 1), wave = tid >> 6, nw = nt >> 6;
  const int q = (B + nt - 1) / nt;                    // entries per thread
  const int lo = min(tid * q, B), hi = min(lo + q, B);
  int local = 0;
  for (int b = lo; b < hi; ++b) local += cnt[b] + 1;
  int incl = local;                                   // inclusive scan inside the wavefront
#pragma unroll
  for (int off = 1; off < kWave; off <<= 1) {
    const int up = __shfl_up(incl, off, kWave);
    if (lane >= off) incl += up;
  }
  if (lane == kWave - 1) part[wave] = incl;
  __syncthreads();
  int before = 0, total = 0;                          // wavefronts before this one, and all of them
  for (int w = 0; w < nw; ++w) {
    const int v = part[w];
    if (w < wave) before += v;
    total += v;
  }
  int run = before + incl - local;
  for (int b = lo; b < hi; ++b) {
    const int gb = cnt[b];
    gamma[b] = gb;
    t_offsets[b] = run;
    run += gb + 1;
  }
  if (tid == 0) t_offsets[B] = total;
}

// sv_estimate_select: the estimates are looked up here (the rule of sv_accept_estimate,
// sv_bins.hpp) instead of being read, which saves the launch in between.
struct EstimateArgs {
  const float* S;
  const float* A;
  const float* edges_s;
  const float* edges_a;
  const float* table;
  int n_s, n_a;
  float* p_hat;          // nullable: the estimates are also written out
  uint8_t* edge_flag;    // nullable
};

// The estimate of key j.  es / ea: the edge arrays (in LDS when they fit).
__device__ __forceinline__ float estimate_of(const EstimateArgs& e, const float* es, const float* ea, int j) {
  const float s = e.S[j], a = e.A[j];
  const float p = e.table[bin_of(s, es, e.n_s) * e.n_a + bin_of(a, ea, e.n_a)];
  if (e.p_hat) e.p_hat[j] = p;
  if (e.edge_flag) e.edge_flag[j] = (near_edge(s, es, e.n_s) || near_edge(a, ea, e.n_a)) ? 1 : 0;
  return p;
}

template <bool FUSED>
__global__ __launch_bounds__(kSelThreads) void select_batch_kernel(
    const float* p_hat, int B, int k, const float* latency, int32_t* gamma, int32_t* t_offsets,
    int32_t* total_M, EstimateArgs est) {
  __shared__ double key_c[kSelMax];     // sort keys, later the running sums E_M
  __shared__ int key_i[kSelMax];        // first the raw estimates (as float bits), then key indices
  __shared__ int part[kSelThreads];
  __shared__ int m_star;
  const int tid = threadIdx.x, nt = blockDim.x;
  const int n = B * k;
  int npad = kWave;                    // a power of two >= max(n, 64)
  while (npad < n) npad <<= 1;

  SV_PHASE_MARK(0)
  // the latencies this lane divides by after the sort: asked for now, so that the
  // memory latency passes behind the sort
  constexpr int kRunMax = kSelMax / kSelThreads;
  const int R = (npad + nt - 1) / nt;                  // keys per lane in the goodput scan
  float lat_run[kRunMax];
#pragma unroll
  for (int j = 0; j < kRunMax; ++j) {
    const int idx = tid * R + j;
    lat_run[j] = (j < R && idx < n) ? latency[idx + 1] : 1.f;
  }
  // estimates into LDS with one round of coalesced loads
  float* p_lds = reinterpret_cast<float*>(key_i);
  if (FUSED) {
    __shared__ float e_lds[kEdgeLds];
    const bool in_lds = stage_edges(e_lds, est.edges_s, est.n_s, est.edges_a, est.n_a);
    const float* es = in_lds ? e_lds : est.edges_s;
    const float* ea = in_lds ? e_lds + est.n_s + 1 : est.edges_a;
    for (int j = tid; j < n; j += nt) p_lds[j] = estimate_of(est, es, ea, j);
  } else {
    for (int j = tid; j < n; j += nt) p_lds[j] = p_hat[j];
  }
  __syncthreads();
  for (int b = tid; b < B; b += nt) {
    double acc = 1.0;
    for (int j = 0; j < k; ++j) {
      acc = acc * clean_p(p_lds[b * k + j]);
      key_c[b * k + j] = acc;
    }
  }
  __syncthreads();
  for (int j = tid; j < npad; j += nt) {
    if (j < n) { key_i[j] = j; } else { key_c[j] = -1.0; key_i[j] = 0x7fffffff; }
  }
  if (tid == 0) m_star = n;
  __syncthreads();

  SV_PHASE_MARK(1)
  // Sort into selection order.  Every sequence's keys are already in order
  // (c is non-increasing along a sequence), so up to kMergeMax keys are merged
  // pairwise, list lengths k, 2k, 4k, ...: a key's new position is its position
  // in its own list plus the number of keys of the partner list that come
  // before it, found by binary search.  Ties between the two lists go to the
  // left one (lower sequence indices), which is the tie order of the keys.
  if (n <= kMergeMax) {
    // ping-pong between the lower and the upper half of the key arrays
    int src = 0, dst = kMergeMax;
    for (int len = k; len < n; len <<= 1) {
      for (int p = tid; p < n; p += nt) {
        const int base = (p / (2 * len)) * (2 * len);
        const int mid = min(n, base + len), end = min(n, base + 2 * len);
        const bool left = p < mid;
        const double c = key_c[src + p];
        int lo = left ? mid : base, hi = left ? end : mid;
        const int first = lo;
        while (lo < hi) {
          const int probe = (lo + hi) >> 1;
          const double v = key_c[src + probe];
          if (left ? (v > c) : (v >= c)) lo = probe + 1; else hi = probe;
        }
        const int q = base + (left ? p - base : p - mid) + (lo - first);
        key_c[dst + q] = c;
        key_i[dst + q] = key_i[src + p];
      }
      __syncthreads();
      const int t = src; src = dst; dst = t;
    }
    if (src != 0) {                              // odd number of rounds: bring the result down
      for (int p = tid; p < n; p += nt) { key_c[p] = key_c[src + p]; key_i[p] = key_i[src + p]; }
      __syncthreads();
    }
  } else {
    // More keys than the second buffer holds: the same merge rounds in place.  Every
    // lane first takes its keys of the round into registers and finds their new
    // positions (reading the old order), then, after a barrier, scatters them.
    for (int len = k; len < n; len <<= 1) {
      double c_reg[kRunMax];
      int i_reg[kRunMax], q_reg[kRunMax];
#pragma unroll
      for (int j = 0; j < kRunMax; ++j) {
        const int p = tid + j * nt;
        q_reg[j] = -1;
        if (p < n) {
          const int base = (p / (2 * len)) * (2 * len);
          const int mid = min(n, base + len), end = min(n, base + 2 * len);
          const bool left = p < mid;
          const double c = key_c[p];
          int lo = left ? mid : base, hi = left ? end : mid;
          const int first = lo;
          while (lo < hi) {
            const int probe = (lo + hi) >> 1;
            const double v = key_c[probe];
            if (left ? (v > c) : (v >= c)) lo = probe + 1; else hi = probe;
          }
          c_reg[j] = c;
          i_reg[j] = key_i[p];
          q_reg[j] = base + (left ? p - base : p - mid) + (lo - first);
        }
      }
      __syncthreads();
#pragma unroll
      for (int j = 0; j < kRunMax; ++j)
        if (q_reg[j] >= 0) { key_c[q_reg[j]] = c_reg[j]; key_i[q_reg[j]] = i_reg[j]; }
      __syncthreads();
    }
  }

  SV_PHASE_MARK(2)
  // First peak of the estimated goodput G_M = E_M / latency[M], G_0 = 0:
  // M* = first M >= 0 with not (G_{M+1} > G_M).  E_M is DEFINED as the running
  // sum in selection order (fp64, one addition after another), so that the
  // integer outputs do not depend on a reduction tree.  Fast path: a parallel
  // scan gives sums E'_M that differ from E_M by at most 2 n u E_M (all terms are
  // non-negative, u = 2^-53); wherever |G'_{M+1} - G'_M| exceeds the resulting
  // bound the comparison is already decided.  Only if an undecided comparison
  // comes before the first decided stop does one lane run the ordered sum.
  // (The bound holds for any summation tree, so lanes may own runs of keys.)
  bool need_exact = false;
  {
    __shared__ double wave_tot[kSelThreads / kWave];
    __shared__ double wave_last_g[kSelThreads / kWave];
    __shared__ int first_stop, first_open;
    if (tid == 0) { first_stop = n; first_open = n; }
    const int lane = tid & (kWave - 1), wave = tid >> 6;
    // every lane owns a run of R consecutive keys (R = 1 up to 1024 keys)
    double e_run[kRunMax];
    double run = 0.0;
#pragma unroll
    for (int j = 0; j < kRunMax; ++j) {
      const int idx = tid * R + j;
      if (j < R) run += (idx < n) ? key_c[idx] : 0.0;
      e_run[j] = run;                              // inclusive inside the run
    }
    double e = run;                                // inclusive scan of the run totals
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
      int lo = __double2loint(e), hi = __double2hiint(e);
      lo = __shfl_up(lo, off, kWave);
      hi = __shfl_up(hi, off, kWave);
      if (lane >= off) e += __hiloint2double(hi, lo);
    }
    if (lane == kWave - 1) wave_tot[wave] = e;
    __syncthreads();
    for (int w = 0; w < wave; ++w) e += wave_tot[w];
    const double base = e - run;                   // E' of everything before this lane's run
    double g_run[kRunMax];                         // G'_{idx+1} of the run's keys
#pragma unroll
    for (int j = 0; j < kRunMax; ++j) {
      const int idx = tid * R + j;
      g_run[j] = (j < R && idx < n) ? (base + e_run[j]) / (double)lat_run[j] : 0.0;
    }
    double g_last = 0.0;                           // G' of the last key of the run
#pragma unroll
    for (int j = 0; j < kRunMax; ++j) if (j == R - 1) g_last = g_run[j];
    if (lane == kWave - 1) wave_last_g[wave] = g_last;
    __syncthreads();
    int lo = __double2loint(g_last), hi = __double2hiint(g_last);
    lo = __shfl_up(lo, 1, kWave);
    hi = __shfl_up(hi, 1, kWave);
    double g_cur = __hiloint2double(hi, lo);                                 // G' of the key before the run
    if (lane == 0) g_cur = (wave == 0) ? 0.0 : wave_last_g[wave - 1];
#pragma unroll
    for (int j = 0; j < kRunMax; ++j) {
      const int idx = tid * R + j;
      if (j < R && idx < n) {
        const double g_nxt = g_run[j];
        const double bound = 8.0 * (double)(n + 2) * 1.1102230246251565e-16 * fmax(g_nxt, g_cur);
        const double d = g_nxt - g_cur;
        if (d < -bound) atomicMin(&first_stop, idx);
        else if (!(d > bound)) atomicMin(&first_open, idx);                  // undecided (or NaN)
        g_cur = g_nxt;
      }
    }
    __syncthreads();
    if (first_open < first_stop) need_exact = true;  // block-uniform
    else if (tid == 0) m_star = first_stop;
  }
  SV_PHASE_MARK(3)
  if (need_exact) {
    // ordered sum by one lane: key_c[M-1] becomes E_M.  The padding keys sort
    // last, so running over whole batches of 16 never touches E_1..E_n.
    __syncthreads();
    if (tid == 0) {
      double E = 0.0;
      for (int j0 = 0; j0 < npad; j0 += 16) {   // batches of loads keep LDS latency off the add chain
        double v[16];
#pragma unroll
        for (int q = 0; q < 16; ++q) v[q] = key_c[j0 + q];
#pragma unroll
        for (int q = 0; q < 16; ++q) { E += v[q]; v[q] = E; }
#pragma unroll
        for (int q = 0; q < 16; ++q) key_c[j0 + q] = v[q];
      }
    }
    __syncthreads();
    for (int M = tid; M < n; M += nt) {
      const double g_cur = (M == 0) ? 0.0 : key_c[M - 1] / (double)latency[M];
      const double g_nxt = key_c[M] / (double)latency[M + 1];
      if (!(g_nxt > g_cur)) atomicMin(&m_star, M);
    }
  }
  __syncthreads();
  SV_PHASE_MARK(4)
  const int M = m_star;
  int* cnt = reinterpret_cast<int*>(key_c);      // the keys are dead: selected tokens per sequence
  for (int b = tid; b < B; b += nt) cnt[b] = 0;
  __syncthreads();
  for (int r = tid; r < M; r += nt) atomicAdd(&cnt[key_i[r] / k], 1);
  if (tid == 0) *total_M = M;
  __syncthreads();
  SV_PHASE_MARK(5)
  offsets_scan(cnt, B, gamma, t_offsets, part);
  SV_PHASE_MARK(6)
}

template <bool FUSED>
__global__ __launch_bounds__(kSelThreads) void select_per_sequence_kernel(
    const float* p_hat, int B, int k, const float* latency, int32_t* gamma, int32_t* t_offsets,
    int32_t* total_M, EstimateArgs est) {
  __shared__ int part[kSelThreads];
  __shared__ int total;
  const int tid = threadIdx.x, nt = blockDim.x;
  if (tid == 0) total = 0;
  if (FUSED) {
    // every estimate is looked up (and written out) first: the search below stops early
    __shared__ float e_lds[kEdgeLds];
    const bool in_lds = stage_edges(e_lds, est.edges_s, est.n_s, est.edges_a, est.n_a);
    const float* es = in_lds ? e_lds : est.edges_s;
    const float* ea = in_lds ? e_lds + est.n_s + 1 : est.edges_a;
    for (int j = tid; j < B * k; j += nt) est.p_hat[j] = estimate_of(est, es, ea, j);
    __threadfence_block();
  }
  __syncthreads();
  int mine = 0;
  for (int b = tid; b < B; b += nt) {
    double acc = 1.0, E = 0.0, best = 0.0;
    int g = 0;
    while (g < k) {
      acc = acc * clean_p(p_hat[b * k + g]);
      const double E_new = E + acc;
      const double good = E_new / (double)latency[g + 1];
      if (!(good > best)) break;
      E = E_new; best = good; ++g;
    }
    gamma[b] = g;
    mine += g;
  }
  if (mine) atomicAdd(&total, mine);
  __syncthreads();
  if (tid == 0) *total_M = total;
  offsets_scan(gamma, B, gamma, t_offsets, part);
}

}  // namespace sv

namespace sv {
// Argument checks and launch shared by sv_select_length and sv_estimate_select.
static int select_checked(const float* p_hat, int B, int k, const float* latency, int n_latency, int mode,
                          int32_t* gamma, int32_t* t_offsets, int32_t* total_M, const EstimateArgs* est,
                          sv_stream_t stream) {
  SV_REQUIRE(mode == SV_BATCH_GREEDY || mode == SV_PER_SEQUENCE, SV_ERR_INVALID_ARG);
  SV_REQUIRE(B >= 0 && k >= 1, SV_ERR_INVALID_ARG);
  SV_REQUIRE(!est || (est->n_s >= 1 && est->n_a >= 1), SV_ERR_INVALID_ARG);
  SV_REQUIRE((long long)B * k <= SV_SELECT_MAX_KEYS, SV_ERR_TOO_LARGE);
  if (B == 0) return SV_OK;
  SV_REQUIRE(n_latency >= (mode == SV_BATCH_GREEDY ? B * k + 1 : k + 1), SV_ERR_INVALID_ARG);
  SV_REQUIRE(p_hat && latency && gamma && t_offsets && total_M, SV_ERR_NULL);
  SV_REQUIRE(is_aligned(p_hat, 4) && is_aligned(latency, 4) && is_aligned(gamma, 4) &&
                 is_aligned(t_offsets, 4) && is_aligned(total_M, 4),
             SV_ERR_ALIGN);
  if (est) {
    SV_REQUIRE(est->S && est->A && est->edges_s && est->edges_a && est->table, SV_ERR_NULL);
    SV_REQUIRE(is_aligned(est->S, 4) && is_aligned(est->A, 4) && is_aligned(est->edges_s, 4) &&
                   is_aligned(est->edges_a, 4) && is_aligned(est->table, 4),
               SV_ERR_ALIGN);
  }
  hipStream_t st = as_stream(stream);
  TapScope tap(SV_KERNEL_SELECT_LENGTH, st);
  // one lane per (padded) key up to the workgroup limit
  int threads = 64;
  while (threads < kSelThreads && threads < B * k) threads <<= 1;
  const EstimateArgs none = {};
  if (mode == SV_BATCH_GREEDY) {
    if (est)
      hipLaunchKernelGGL(select_batch_kernel<true>, dim3(1), dim3(threads), 0, st, p_hat, B, k, latency, gamma,
                         t_offsets, total_M, *est);
    else
      hipLaunchKernelGGL(select_batch_kernel<false>, dim3(1), dim3(threads), 0, st, p_hat, B, k, latency, gamma,
                         t_offsets, total_M, none);
  } else {
    if (est)
      hipLaunchKernelGGL(select_per_sequence_kernel<true>, dim3(1), dim3(kSelThreads), 0, st, p_hat, B, k, latency,
                         gamma, t_offsets, total_M, *est);
    else
      hipLaunchKernelGGL(select_per_sequence_kernel<false>, dim3(1), dim3(kSelThreads), 0, st, p_hat, B, k, latency,
                         gamma, t_offsets, total_M, none);
  }
  return launch_status();
}
}  // namespace sv

extern "C" int sv_select_length(const float* p_hat, int B, int k, const float* latency, int n_latency,
                                int mode, int32_t* gamma, int32_t* t_offsets, int32_t* total_M,
                                sv_stream_t stream) {
  return sv::select_checked(p_hat, B, k, latency, n_latency, mode, gamma, t_offsets, total_M, nullptr, stream);
}

extern "C" int sv_estimate_select(const float* S, const float* A, int B, int k,
                                  const float* edges_s, int n_s, const float* edges_a, int n_a,
                                  const float* table, const float* latency, int n_latency, int mode,
                                  float* p_hat, uint8_t* edge_flag_or_null,
                                  int32_t* gamma, int32_t* t_offsets, int32_t* total_M, sv_stream_t stream) {
  const sv::EstimateArgs est{S, A, edges_s, edges_a, table, n_s, n_a, p_hat, edge_flag_or_null};
  return sv::select_checked(p_hat, B, k, latency, n_latency, mode, gamma, t_offsets, total_M, &est, stream);
}
