// Host-side helpers of the C ABI: argument checks, launch checks and the
// layout of the caller-provided device workspace.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/sv.h"

namespace sv {

struct Plan;

constexpr int kChunk = 8192;          // vocabulary entries per sampling chunk
constexpr size_t kWsAlign = 256;
constexpr int kMaxSplit = 8;          // a row may be swept by up to 8 workgroups
// SV_FLAG_NEAR_CDF_EDGE: the sampling threshold lies within kCdfEdgeRel * W + kCdfEdgeAbs of an
// edge of the chosen token's CDF interval.  The absolute part is the resolution of the dense
// path's own arithmetic: its probabilities are fp32 numbers with a relative error of at most
// 2.5e-7 each (row normaliser 1e-7, exponent rounding and v_exp_f32 1.5e-7), so a cumulative
// sum of max(0, p_t - p_d) is off by at most 2.5e-7 * (P_t + P_d)(<= v) <= 5e-7, and so is the
// threshold u' * W: 1e-6 between them.  Compacted supports carry fp64 probabilities: no such part.
constexpr double kCdfEdgeRel = 1e-6;
constexpr double kCdfEdgeAbs = 1e-6;

inline hipStream_t as_stream(sv_stream_t s) { return reinterpret_cast<hipStream_t>(s); }

inline int elem_bytes(int dtype) { return dtype == SV_F32 ? 4 : (dtype == SV_BF16 ? 2 : 0); }

inline bool is_aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

inline int n_chunks(int V) { return (V + kChunk - 1) / kChunk; }

// What sv_row_stats leaves in the workspace for sv_verify_sample_chained: which
// call wrote the draft normalisers that follow it.
struct alignas(16) ChainHeader {
  uint64_t z_d, x, cut_d;    // device addresses the statistics pass was given (cut_d: 0 without warps)
  int32_t B, k, V, dtype;
  uint32_t scale_bits;       // bit pattern of the draft's exponent scale fl32(log2(e) / T)
  uint32_t magic;
};
constexpr uint32_t kChainMagic = 0x53564348u;

// Workspace carve-up for sv_verify_sample.  All offsets are multiples of 256.
struct VerifyWs {
  double* s_t;        // [B*(k+1)*kMaxSplit] partial sums relative to c(m) of each target row
  double* s_d;        // [B*k*kMaxSplit]     same for draft rows
  float* m_t;         // [B*(k+1)*kMaxSplit] partial maxima
  float* m_d;         // [B*k*kMaxSplit]
  float* zx_t;        // [B*k] target logit of the drafted token
  float* zx_d;        // [B*k] draft logit of the drafted token
  double* mass_r;     // [B*C] residual mass of each chunk of the sampling row
  double* mass_t;     // [B*C] target mass of each chunk of the sampling row
  Plan* plan;          // [B] per-sequence sampling plan (verify_sample.hip)
  // written by sv_row_stats, read by sv_verify_sample_chained
  ChainHeader* chain;  // [1]
  double* chain_s;     // [B*k] sum relative to c(m) of each whole draft row
  float* chain_m;      // [B*k] maximum of each draft row
  float* chain_zx;     // [B*k] draft logit of the drafted token (NaN: token out of range)
  size_t bytes;
};

inline size_t ws_round(size_t n) { return (n + kWsAlign - 1) / kWsAlign * kWsAlign; }

inline VerifyWs carve_verify_ws(void* base, int B, int k, int V) {
  VerifyWs w;
  char* p = static_cast<char*>(base);
  size_t off = 0;
  const size_t rt = (size_t)B * (k + 1), rd = (size_t)B * k, bc = (size_t)B * n_chunks(V);
  auto take = [&](size_t bytes) { char* q = p ? p + off : nullptr; off += ws_round(bytes); return q; };
  w.s_t = reinterpret_cast<double*>(take(rt * kMaxSplit * 8));
  w.s_d = reinterpret_cast<double*>(take(rd * kMaxSplit * 8));
  w.m_t = reinterpret_cast<float*>(take(rt * kMaxSplit * 4));
  w.m_d = reinterpret_cast<float*>(take(rd * kMaxSplit * 4));
  w.zx_t = reinterpret_cast<float*>(take(rd * 4));
  w.zx_d = reinterpret_cast<float*>(take(rd * 4));
  w.mass_r = reinterpret_cast<double*>(take(bc * 8));
  w.mass_t = reinterpret_cast<double*>(take(bc * 8));
  w.plan = reinterpret_cast<Plan*>(take((size_t)B * 32));
  w.chain = reinterpret_cast<ChainHeader*>(take(sizeof(ChainHeader)));
  w.chain_s = reinterpret_cast<double*>(take(rd * 8));
  w.chain_m = reinterpret_cast<float*>(take(rd * 4));
  w.chain_zx = reinterpret_cast<float*>(take(rd * 4));
  w.bytes = off;
  return w;
}

inline int launch_status() { return hipGetLastError() == hipSuccess ? SV_OK : SV_ERR_LAUNCH; }

// Optional hipEvent pair recorded right before / after a kernel (api.hip).
struct TimingTap {
  hipEvent_t start, stop;
};
TimingTap timing_tap(int kernel);      // the pair set for `kernel` (nulls when none); safe from any thread

struct TapScope {           // records start on construction, stop on destruction
  hipStream_t st;
  hipEvent_t stop;
  TapScope(int kernel, hipStream_t s) : st(s), stop(nullptr) {
    const TimingTap tap = timing_tap(kernel);
    stop = tap.stop;
    if (tap.start) (void)hipEventRecord(tap.start, st);
  }
  ~TapScope() {
    if (stop) (void)hipEventRecord(stop, st);
  }
};

}  // namespace sv

#define SV_REQUIRE(cond, code) \
  do {                         \
    if (!(cond)) return (code); \
  } while (0)
