// Device-side building blocks shared by the SV kernels (gfx950 only).
//
//  * 128-bit streaming loads of bf16 / fp32 logits and their unpacking
//  * the per-lane online (max, sum-exp) accumulator in the base-2 domain
//  * wavefront (64-lane) and workgroup reductions
//  * Philox-4x32-10 for the speculative-sampling uniforms
//
// A row's normaliser is carried as the pair (m, s): m = the row maximum in raw
// logit units and s = sum_v 2^(z_v * L - c(m)), c(m) = max(fl32(m * L), -2^30),
// where L is log2(e) / T rounded to fp32 (T = sampling temperature of the
// tensor, 1 unless a warped entry point says otherwise; L32 is the T = 1 value).
// Because L T / log2(e) = 1 + tau1 with |tau1| < 6e-8 (1.33e-8 for L32) the sum
// is the soft-max normaliser at a temperature off by that factor; the fp64
// epilogue removes the first-order effect around the row maximum
// (lse_from_ms), leaving an error below |tau1| * (H - H_inf) of the row.
//
// Range of the logits.  2^(z L - c) is formed with one fused multiply-add, so it
// is right for any z as long as the part of m * L that fp32 drops from c stays a
// small exponent: |c| <= 2^30 keeps it within +-32.  Hence the floor of c: an
// entry with z L < -2^30 (a finite stand-in for -inf such as -1e30, or the
// lowest finite number of the storage type) carries no mass, exactly like
// -inf, and a row without any entry above the floor is a bad row.  A row whose
// maximum has m * L > 2^30 is a bad row as well.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sv {

constexpr int kWave = 64;
constexpr float kL32 = 1.44269502162933349609375f;          // fl32(log2 e)
constexpr double kLog2e = 1.4426950408889634073599246810019;  // log2 e
constexpr double kLn2 = 0.69314718055994530941723212145818;
constexpr double kTauMinus1 = (double)kL32 / kLog2e - 1.0;   // ~ +1.33e-8
constexpr float kRefFloor = -1073741824.f;                    // -2^30: lowest reference c(m)
constexpr float kRefCeil = 1073741824.f;                      // 2^30: highest usable reference

// Exponent scale of one logit tensor: 2^(z L) = e^((z / T) (1 + tau1)).
struct Scale {
  float L;        // fl32(log2(e) / T)
  double l_lo;    // log2(e) / T - L, the part of the scale that fp32 drops
  double inv_t;   // 1 / T
  double tau1;    // L T / log2(e) - 1
};

// T = 1: the constants every unwarped kernel folds at compile time.
__host__ __device__ constexpr Scale unit_scale() {
  return Scale{kL32, kLog2e - (double)kL32, 1.0, kTauMinus1};
}

// Scale of a caller-given temperature; false outside [1e-3, 1e3] (or NaN).
inline bool scale_of(float temperature, Scale* sc) {
  if (!(temperature >= 1e-3f && temperature <= 1e3f)) return false;
  const double t = (double)temperature, l = kLog2e / t;
  sc->L = (float)l;
  sc->l_lo = l - (double)sc->L;
  sc->inv_t = 1.0 / t;
  sc->tau1 = (double)sc->L * t / kLog2e - 1.0;
  return true;
}

// Entries below a row's cutoff are outside the warped distribution's support;
// NaN entries stay NaN so that a bad row is still seen as one.
__device__ __forceinline__ float cut_below(float z, float cut) { return z < cut ? -INFINITY : z; }

enum { DT_F32 = 0, DT_BF16 = 1 };

template <int DT> struct Elem;
template <> struct Elem<DT_F32> { static constexpr int bytes = 4; static constexpr int per_vec = 4; };
template <> struct Elem<DT_BF16> { static constexpr int bytes = 2; static constexpr int per_vec = 8; };

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));   // one 128-bit load

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// v_exp_f32: 2^x, no denormal fix-ups (results below 2^-126 flush to zero, which
// is what a vanishing probability mass should do here).
__device__ __forceinline__ float exp2_fast(float x) { return __builtin_amdgcn_exp2f(x); }

// One scalar logit of a row.
template <int DT>
__device__ __forceinline__ float load_elem(const void* row, int v) {
  if (DT == DT_F32) return reinterpret_cast<const float*>(row)[v];
  uint32_t h = reinterpret_cast<const uint16_t*>(row)[v];
  return __uint_as_float(h << 16);
}

// Unpack one 16-byte vector into per_vec floats.
template <int DT>
__device__ __forceinline__ void unpack(const u32x4& q, float (&f)[Elem<DT>::per_vec]) {
  if constexpr (DT == DT_F32) {
    f[0] = __uint_as_float(q.x); f[1] = __uint_as_float(q.y);
    f[2] = __uint_as_float(q.z); f[3] = __uint_as_float(q.w);
  } else {
    f[0] = bf16_lo(q.x); f[1] = bf16_hi(q.x);
    f[2] = bf16_lo(q.y); f[3] = bf16_hi(q.y);
    f[4] = bf16_lo(q.z); f[5] = bf16_hi(q.z);
    f[6] = bf16_lo(q.w); f[7] = bf16_hi(q.w);
  }
}

__device__ __forceinline__ bool aligned16(const void* p) {
  return (reinterpret_cast<uintptr_t>(p) & 15u) == 0;
}

// ---------------------------------------------------------------------------
// online (max, sum 2^(z L - c)) accumulator, one per lane
// ---------------------------------------------------------------------------
struct Online {
  float m;   // running maximum (raw units); -inf before the first element
  float c;   // max(fl32(m * L), kRefFloor)
  float s;   // sum of 2^(z*L - c) so far

  __device__ __forceinline__ void init() { m = -INFINITY; c = kRefFloor; s = 0.f; }

  template <int N>
  __device__ __forceinline__ void add(const float (&z)[N], const float L = kL32) {
    float mx = m;
#pragma unroll
    for (int j = 0; j + 1 < N; j += 2) mx = fmaxf(fmaxf(mx, z[j]), z[j + 1]);   // v_max3_f32
    if (N & 1) mx = fmaxf(mx, z[N - 1]);
    const float cn = fmaxf(mx * L, kRefFloor);
    const float scale = exp2_fast(c - cn);
    float e[N];
#pragma unroll
    for (int j = 0; j < N; ++j) e[j] = exp2_fast(__builtin_fmaf(z[j], L, -cn));
    // pairwise tree so that no single chain carries all roundings
    float t = 0.f;
    if constexpr (N == 8) {
      t = ((e[0] + e[1]) + (e[2] + e[3])) + ((e[4] + e[5]) + (e[6] + e[7]));
    } else if constexpr (N == 4) {
      t = (e[0] + e[1]) + (e[2] + e[3]);
    } else {
#pragma unroll
      for (int j = 0; j < N; ++j) t += e[j];
    }
    s = __builtin_fmaf(s, scale, t);
    m = mx;
    c = cn;
  }

  __device__ __forceinline__ void add1(float z, const float L = kL32) {
    const float mx = fmaxf(m, z);
    const float cn = fmaxf(mx * L, kRefFloor);
    s = __builtin_fmaf(s, exp2_fast(c - cn), exp2_fast(__builtin_fmaf(z, L, -cn)));
    m = mx;
    c = cn;
  }
};

// A row's normaliser: exact maximum m and fp64 sum s relative to c(m).
struct MS {
  float m;
  double s;
};

__device__ __forceinline__ float ref_of(float m, const float L = kL32) { return fmaxf(m * L, kRefFloor); }

__device__ __forceinline__ double shfl_xor_f64(double v, int mask) {
  int lo = __double2loint(v), hi = __double2hiint(v);
  lo = __shfl_xor(lo, mask, kWave);
  hi = __shfl_xor(hi, mask, kWave);
  return __hiloint2double(hi, lo);
}

__device__ __forceinline__ float wave_max_f32(float v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, kWave));
  return v;
}

__device__ __forceinline__ double wave_sum_f64(double v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v += shfl_xor_f64(v, off);
  return v;
}

// Scratch for the workgroup reductions below (up to 16 waves).
struct BlockScratch {
  float f[16];
  double d[16];
};

// Workgroup sum of fp64 partials in a fixed order; result in every thread.
__device__ __forceinline__ double block_sum_f64(double v, BlockScratch& sm) {
  v = wave_sum_f64(v);
  const int wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
  if ((threadIdx.x & 63) == 0) sm.d[wave] = v;
  __syncthreads();
  double r = 0.0;
  for (int w = 0; w < nw; ++w) r += sm.d[w];
  __syncthreads();
  return r;
}

__device__ __forceinline__ float block_max_f32(float v, BlockScratch& sm) {
  v = wave_max_f32(v);
  const int wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
  if ((threadIdx.x & 63) == 0) sm.f[wave] = v;
  __syncthreads();
  float r = sm.f[0];
  for (int w = 1; w < nw; ++w) r = fmaxf(r, sm.f[w]);
  __syncthreads();
  return r;
}

// Workgroup merge of the per-lane accumulators of NR rows at once; results
// valid in every thread after a single barrier.  Inside a wavefront every lane
// rescales its sum to the wavefront's reference (a factor 2^(c_lane - c_wave)
// <= 1 from v_exp_f32) and the sums are added in fp64; the per-wavefront
// pairs go through LDS and every thread folds them in the same fixed order.
template <int NR>
struct MergeScratch {
  float m[NR][16];
  double s[NR][16];
};

template <int NR>
__device__ __forceinline__ void block_merge(const Online (&o)[NR], MergeScratch<NR>& sm, MS (&out)[NR],
                                            const float L = kL32) {
  const int wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
#pragma unroll
  for (int r = 0; r < NR; ++r) {
    const float mw = wave_max_f32(o[r].m);
    const double sw = wave_sum_f64((double)o[r].s * (double)exp2_fast(o[r].c - ref_of(mw, L)));
    if ((threadIdx.x & 63) == 0) { sm.m[r][wave] = mw; sm.s[r][wave] = sw; }
  }
  __syncthreads();
#pragma unroll
  for (int r = 0; r < NR; ++r) {
    float m = sm.m[r][0];
    for (int w = 1; w < nw; ++w) m = fmaxf(m, sm.m[r][w]);
    const float cr = ref_of(m, L);
    double acc = 0.0;
    for (int w = 0; w < nw; ++w) acc += sm.s[r][w] * (double)exp2_fast(ref_of(sm.m[r][w], L) - cr);
    out[r].m = m;
    out[r].s = acc;
  }
}

// Row normaliser in fp64 from (m, s):  log2-domain kappa = c(m) + log2 s is the
// log2 of sum_v 2^(z_v L); the natural-log LSE of the row z / T follows after
// removing the temperature offset around the maximum.  Bad rows (NaN, +inf, no
// finite entry) give NaN.
__device__ __forceinline__ double lse_from_ms(const MS& r, const Scale sc = unit_scale()) {
  if (!(r.s > 0.0) || !isfinite(r.s) || !isfinite(r.m) || ref_of(r.m, sc.L) > kRefCeil) return __builtin_nan("");
  const double kappa = (double)ref_of(r.m, sc.L) + log2(r.s);
  return kappa * kLn2 - sc.tau1 * ((double)r.m * sc.inv_t);
}

// log2 of sum_v 2^(z_v L): the normaliser that makes 2^(z L - kappa) sum to
// one.  Those probabilities are the soft-max of z / T at temperature 1 + tau1;
// entry v deviates from the exact one by a relative tau1 * (y_v - E_p[y]),
// y = z / T (1.33e-8 per unit for L32).
__device__ __forceinline__ double kappa_l32(const MS& r, const float L = kL32) {
  return (double)ref_of(r.m, L) + log2(r.s);
}

// Fold `n` partial normalisers (consecutive entries).
__device__ __forceinline__ MS fold_parts(const float* m, const double* s, int n, const float L = kL32) {
  MS r;
  r.m = m[0];
  for (int p = 1; p < n; ++p) r.m = fmaxf(r.m, m[p]);
  const float cr = ref_of(r.m, L);
  r.s = 0.0;
  for (int p = 0; p < n; ++p) r.s += s[p] * (double)exp2_fast(ref_of(m[p], L) - cr);
  return r;
}

// The same for the `split` <= kMaxParts parts of a row held in global memory:
// all loads are issued before the first use (the loop above would pay one
// memory latency per part).
constexpr int kMaxParts = 8;

__device__ __forceinline__ MS fold_row_parts(const float* m, const double* s, int split, const float L = kL32) {
  float mp[kMaxParts];
  double sp[kMaxParts];
#pragma unroll
  for (int p = 0; p < kMaxParts; ++p) {
    const bool on = p < split;
    mp[p] = on ? m[p] : -INFINITY;
    sp[p] = on ? s[p] : 0.0;
  }
  MS r;
  r.m = mp[0];
#pragma unroll
  for (int p = 1; p < kMaxParts; ++p) r.m = fmaxf(r.m, mp[p]);
  const float cr = ref_of(r.m, L);
  r.s = 0.0;
#pragma unroll
  for (int p = 0; p < kMaxParts; ++p) r.s += sp[p] * (double)exp2_fast(ref_of(mp[p], L) - cr);   // absent parts add 0
  return r;
}

// ---------------------------------------------------------------------------
// Sweep of part `part` of `split` of one row: online accumulation by the whole
// workgroup.  Parts are contiguous runs of whole 16-byte vectors (the last one
// also takes the scalar tail); rows that do not start on 16 bytes are split by
// elements and read with scalar loads.
// ---------------------------------------------------------------------------
// NT: the row is not read again soon (non-temporal loads).  U: vectors in flight per lane.
template <int DT, bool CUT = false, bool NT = true, int U = 4>
__device__ __forceinline__ void sweep_online(const void* row, int V, int part, int split, Online& acc,
                                             const float L = kL32, const float cut = -INFINITY) {
  constexpr int EPV = Elem<DT>::per_vec;
  const int tid = threadIdx.x, nt = blockDim.x;
  auto add_vec = [&](const u32x4& q) {
    float f[EPV];
    unpack<DT>(q, f);
    if (CUT) {
#pragma unroll
      for (int j = 0; j < EPV; ++j) f[j] = cut_below(f[j], cut);
    }
    acc.add(f, L);
  };
  auto add_one = [&](int v) {
    const float z = load_elem<DT>(row, v);
    acc.add1(CUT ? cut_below(z, cut) : z, L);
  };
  if (aligned16(row)) {
    const u32x4* p = reinterpret_cast<const u32x4*>(row);
    const int nvec = V / EPV;
    const int per = (nvec + split - 1) / split;
    const int end = min(nvec, (part + 1) * per);
    int i = part * per + tid;
    auto load = [&](int j) { return NT ? __builtin_nontemporal_load(p + j) : p[j]; };
    for (; i + (U - 1) * nt < end; i += U * nt) {
      u32x4 q[U];
#pragma unroll
      for (int u = 0; u < U; ++u) q[u] = load(i + u * nt);
#pragma unroll
      for (int u = 0; u < U; ++u) add_vec(q[u]);
    }
    if (i < end) {
      // the last, partial round: its loads go out together as well (one trip to memory, not one per vector)
      u32x4 q[U - 1];
#pragma unroll
      for (int u = 0; u < U - 1; ++u)
        if (i + u * nt < end) q[u] = load(i + u * nt);
#pragma unroll
      for (int u = 0; u < U - 1; ++u)
        if (i + u * nt < end) add_vec(q[u]);
    }
    if (part == split - 1)
      for (int v = nvec * EPV + tid; v < V; v += nt) add_one(v);
  } else {
    const int per = (V + split - 1) / split;
    const int end = min(V, (part + 1) * per);
    for (int v = part * per + tid; v < end; v += nt) add_one(v);
  }
}

// ---------------------------------------------------------------------------
// Visit elements [v0, v1) of one row (PAIR = false) or of two rows at the same
// vocabulary index (PAIR = true) with the whole workgroup: f(v, za, zb).
// Vector loads when both rows start on 16 bytes and v0 is a vector multiple.
// ---------------------------------------------------------------------------
template <int DT, bool PAIR, int UNROLL = 2, class F>
__device__ __forceinline__ void visit_range(const void* a, const void* b, int v0, int v1, F&& f) {
  constexpr int EPV = Elem<DT>::per_vec;
  const int tid = threadIdx.x, nt = blockDim.x;
  const bool vec = aligned16(a) && (!PAIR || aligned16(b)) && (v0 % EPV == 0);
  if (vec) {
    const u32x4* pa = reinterpret_cast<const u32x4*>(a);
    const u32x4* pb = reinterpret_cast<const u32x4*>(b);
    const int i1 = v1 / EPV;
    int i = v0 / EPV + tid;
    for (; i + (UNROLL - 1) * nt < i1; i += UNROLL * nt) {      // UNROLL vector (pairs) in flight per lane
      u32x4 qa[UNROLL], qb[UNROLL];
#pragma unroll
      for (int u = 0; u < UNROLL; ++u) {
        qa[u] = pa[i + u * nt];
        qb[u] = PAIR ? pb[i + u * nt] : qa[u];
      }
#pragma unroll
      for (int u = 0; u < UNROLL; ++u) {
        float fa[EPV], fb[EPV];
        unpack<DT>(qa[u], fa); unpack<DT>(qb[u], fb);
#pragma unroll
        for (int j = 0; j < EPV; ++j) f((i + u * nt) * EPV + j, fa[j], fb[j]);
      }
    }
    for (; i < i1; i += nt) {
      const u32x4 qa = pa[i];
      u32x4 qb = qa;
      if (PAIR) qb = pb[i];
      float fa[EPV], fb[EPV];
      unpack<DT>(qa, fa); unpack<DT>(qb, fb);
#pragma unroll
      for (int j = 0; j < EPV; ++j) f(i * EPV + j, fa[j], fb[j]);
    }
    for (int v = i1 * EPV + tid; v < v1; v += nt) {
      const float za = load_elem<DT>(a, v);
      f(v, za, PAIR ? load_elem<DT>(b, v) : za);
    }
  } else {
    for (int v = v0 + tid; v < v1; v += nt) {
      const float za = load_elem<DT>(a, v);
      f(v, za, PAIR ? load_elem<DT>(b, v) : za);
    }
  }
}

// ---------------------------------------------------------------------------
// Philox-4x32-10 (Salmon et al., SC'11), written for this library
// ---------------------------------------------------------------------------
struct U4 { uint32_t w[4]; };

__device__ __forceinline__ U4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                            uint32_t k0, uint32_t k1) {
  constexpr uint32_t MUL_A = 0xD2511F53u, MUL_B = 0xCD9E8D57u;
  constexpr uint32_t WEYL_A = 0x9E3779B9u, WEYL_B = 0xBB67AE85u;
#pragma unroll
  for (int round = 0; round < 10; ++round) {
    const uint32_t a_hi = __umulhi(MUL_A, c0), a_lo = MUL_A * c0;
    const uint32_t b_hi = __umulhi(MUL_B, c2), b_lo = MUL_B * c2;
    const uint32_t n0 = b_hi ^ c1 ^ k0;
    const uint32_t n2 = a_hi ^ c3 ^ k1;
    c0 = n0; c1 = b_lo; c2 = n2; c3 = a_lo;
    k0 += WEYL_A; k1 += WEYL_B;
  }
  U4 r;
  r.w[0] = c0; r.w[1] = c1; r.w[2] = c2; r.w[3] = c3;
  return r;
}

__device__ __forceinline__ double unit_from_word(uint32_t w) {
  return ((double)(w >> 8) + 0.5) * (1.0 / 16777216.0);
}

}  // namespace sv
