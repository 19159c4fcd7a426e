// sv_row_stats: draft/companion indicators of Speculative Verification
// (Sec. 4.2 of the SV paper and the appendix definitions of S and A).
//
// One workgroup per (sequence, position).  Sweep 1 streams the draft row and
// the companion row together with 128-bit loads and keeps one online
// (max, sum-exp) accumulator per row and lane.  S = sum_v min(P_d, P_c) needs
// both normalisers before the element-wise comparison, so sweep 2 reads the
// pair again (served from L2 / Infinity Cache when the workgroup's pair is
// still resident there) and accumulates
//     min(P_d, P_c) = 2^min(a_d, a_c),  a = z * L32 - kappa   (one exp per entry)
// and, on request, KL(P_d || P_c) = ln2 * sum_v P_d (a_d - a_c).
// A = min(1, P_c(x) / P_d(x)) is a scalar epilogue in fp64.
// Algorithmic HBM traffic: 2 * V * elem_size bytes per workgroup.
#include "sv_device.hpp"
#include "sv_host.hpp"

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
  uint32_t* flags;    // nullable
};

// Online sweep of two rows at once (more independent loads in flight).
template <int DT>
__device__ __forceinline__ void sweep_online_pair(const void* ra, const void* rb, int V,
                                                  Online& acc_a, Online& acc_b) {
  constexpr int EPV = Elem<DT>::per_vec;
  const int tid = threadIdx.x, nt = blockDim.x;
  if (aligned16(ra) && aligned16(rb)) {
    const u32x4* pa = reinterpret_cast<const u32x4*>(ra);
    const u32x4* pb = reinterpret_cast<const u32x4*>(rb);
    const int nvec = V / EPV;
    int i = tid;
    for (; i + nt < nvec; i += 2 * nt) {
      const u32x4 a0 = pa[i], b0 = pb[i], a1 = pa[i + nt], b1 = pb[i + nt];
      float f[EPV];
      unpack<DT>(a0, f); acc_a.add(f);
      unpack<DT>(b0, f); acc_b.add(f);
      unpack<DT>(a1, f); acc_a.add(f);
      unpack<DT>(b1, f); acc_b.add(f);
    }
    for (; i < nvec; i += nt) {
      const u32x4 a0 = pa[i], b0 = pb[i];
      float f[EPV];
      unpack<DT>(a0, f); acc_a.add(f);
      unpack<DT>(b0, f); acc_b.add(f);
    }
    for (int v = nvec * EPV + tid; v < V; v += nt) {
      acc_a.add1(load_elem<DT>(ra, v));
      acc_b.add1(load_elem<DT>(rb, v));
    }
  } else {
    for (int v = tid; v < V; v += nt) {
      acc_a.add1(load_elem<DT>(ra, v));
      acc_b.add1(load_elem<DT>(rb, v));
    }
  }
}

template <int DT, bool WITH_KL>
__global__ __launch_bounds__(kStatsThreads) void row_stats_kernel(StatsArgs a) {
  __shared__ BlockScratch sm;
  const int pair = blockIdx.x;                       // b * k + i
  const size_t row_bytes = (size_t)a.V * Elem<DT>::bytes;
  const void* rd = static_cast<const char*>(a.z_d) + pair * row_bytes;
  const void* rc = static_cast<const char*>(a.z_c) + pair * row_bytes;

  Online od, oc;
  od.init();
  oc.init();
  sweep_online_pair<DT>(rd, rc, a.V, od, oc);
  const MS msd = block_merge(od, sm);
  const MS msc = block_merge(oc, sm);
  const double lse_d = lse_from_ms(msd), lse_c = lse_from_ms(msc);
  const bool bad = isnan(lse_d) || isnan(lse_c);

  double S = __builtin_nan(""), KL = __builtin_nan("");
  if (!bad) {
    // kappa = log2-domain normaliser consistent with the L32 exponent scale,
    // split into an fp32 head and a tail.  With a = z*L32 - head:  P_d = f_d 2^(a_d),  P_c = f_d 2^(a_c + delta),
    // f_d = 2^(-tail_d), delta = tail_d - tail_c, so one scalar factor at the
    // end removes the rounding of both heads.
    const double kappa_d = kappa_l32(msd), kappa_c = kappa_l32(msc);
    const float kd = (float)kappa_d, kc = (float)kappa_c;
    const double tail_d = kappa_d - (double)kd, tail_c = kappa_c - (double)kc;
    const float delta = (float)(tail_d - tail_c);
    float acc_s = 0.f, acc_kl = 0.f;
    visit_range<DT, true>(rd, rc, 0, a.V, [&](int, float zd, float zc) {
      const float ad = __builtin_fmaf(zd, kL32, -kd);
      const float ac = __builtin_fmaf(zc, kL32, -kc) + delta;
      if (WITH_KL) {
        const float pd = exp2_fast(ad);
        acc_s += (ad <= ac) ? pd : exp2_fast(ac);
        if (pd > 0.f) acc_kl = __builtin_fmaf(pd, ad - ac, acc_kl);
      } else {
        acc_s += exp2_fast(fminf(ad, ac));
      }
    });
    const double f_d = exp2(-tail_d);
    S = f_d * block_sum_f64((double)acc_s, sm);
    if (WITH_KL) KL = f_d * kLn2 * block_sum_f64((double)acc_kl, sm);
  }

  if (threadIdx.x == 0) {
    uint32_t fl = bad ? SV_FLAG_BAD_ROW : 0u;
    double A = __builtin_nan("");
    if (!bad) {
      const int tok = a.x[pair];
      if (tok < 0 || tok >= a.V) {
        fl |= SV_FLAG_BAD_TOKEN;
      } else {
        const double ld = (double)load_elem<DT>(rd, tok) - lse_d;
        const double lc = (double)load_elem<DT>(rc, tok) - lse_c;
        A = (ld == -INFINITY) ? 1.0 : fmin(1.0, exp(lc - ld));
      }
    }
    a.lse_d[pair] = (float)lse_d;
    a.lse_c[pair] = (float)lse_c;
    a.S[pair] = (float)S;
    a.A[pair] = (float)A;
    if (WITH_KL) a.kl[pair] = (float)KL;
    if (a.flags) a.flags[pair] = fl;
  }
}

}  // namespace sv

extern "C" int sv_row_stats(const void* z_d, const void* z_c, const int32_t* x,
                            int B, int k, int V, int dtype,
                            float* lse_d, float* lse_c, float* S, float* A,
                            float* kl_or_null, uint32_t* flags_or_null,
                            void* ws, size_t ws_bytes, sv_stream_t stream) {
  using namespace sv;
  SV_REQUIRE(dtype == SV_F32 || dtype == SV_BF16, SV_ERR_DTYPE);
  SV_REQUIRE(B >= 0 && k >= 1 && V >= 1, SV_ERR_INVALID_ARG);
  SV_REQUIRE((long long)B * k <= 0x7fffffffLL, SV_ERR_TOO_LARGE);
  if (B == 0) return SV_OK;
  SV_REQUIRE(z_d && z_c && x && lse_d && lse_c && S && A, SV_ERR_NULL);
  const int eb = elem_bytes(dtype);
  SV_REQUIRE(is_aligned(z_d, eb) && is_aligned(z_c, eb), SV_ERR_ALIGN);
  SV_REQUIRE(is_aligned(x, 4) && is_aligned(lse_d, 4) && is_aligned(lse_c, 4) && is_aligned(S, 4) &&
                 is_aligned(A, 4) && is_aligned(kl_or_null, 4) && is_aligned(flags_or_null, 4),
             SV_ERR_ALIGN);
  SV_REQUIRE(ws && is_aligned(ws, kWsAlign) && ws_bytes >= sv_workspace_bytes(B, k, V, dtype),
             SV_ERR_WORKSPACE);
  StatsArgs a{z_d, z_c, x, B, k, V, lse_d, lse_c, S, A, kl_or_null, flags_or_null};
  const dim3 grid(B * k), block(kStatsThreads);
  hipStream_t st = as_stream(stream);
  TapScope tap(SV_KERNEL_ROW_STATS, st);
  if (dtype == SV_F32) {
    if (kl_or_null) hipLaunchKernelGGL((row_stats_kernel<DT_F32, true>), grid, block, 0, st, a);
    else hipLaunchKernelGGL((row_stats_kernel<DT_F32, false>), grid, block, 0, st, a);
  } else {
    if (kl_or_null) hipLaunchKernelGGL((row_stats_kernel<DT_BF16, true>), grid, block, 0, st, a);
    else hipLaunchKernelGGL((row_stats_kernel<DT_BF16, false>), grid, block, 0, st, a);
  }
  return launch_status();   // the tap's stop event is recorded on scope exit
}
