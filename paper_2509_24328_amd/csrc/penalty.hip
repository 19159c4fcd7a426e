// sv_repetition_penalty: the repetition penalty of the sampling hyper-parameters
// (appendix table of the SV paper; the table gives the value, the operation is
// the usual logits processor): every token of a position's history has its
// logit divided by theta if it is positive and multiplied by theta otherwise,
// once per distinct token, in place, before temperature / top-k / top-p.
// The history of position i of a sequence is the sequence's context plus, when
// the drafted tokens are given, those drafted before i.
//
// One workgroup per logit row.  Every lane first reads the logits of its share
// of the history (up to 16 tokens per lane, kept in registers), the workgroup
// meets at a barrier, then every lane writes the penalised values: all reads of
// a row happen before any write to it, so a token that occurs twice is read
// twice unpenalised and written twice with the same value.  A few thousand
// scattered 2- or 4-byte accesses per row: latency-bound, no bandwidth to speak of.
// Arithmetic: float32 multiply / correctly rounded float32 divide; bfloat16
// storage rounds to nearest-even.
#include "sv_device.hpp"
#include "sv_host.hpp"

namespace sv {

constexpr int kPenaltyThreads = 256;
constexpr int kPenaltyPerLane = SV_PENALTY_MAX_TOKENS / kPenaltyThreads;

template <int DT>
__device__ __forceinline__ void store_elem(void* row, int v, float z) {
  if (DT == DT_F32) {
    reinterpret_cast<float*>(row)[v] = z;
    return;
  }
  const uint32_t u = __float_as_uint(z);
  uint16_t h;
  if (z != z) h = (uint16_t)((u >> 16) | 0x0040u);                        // NaN stays NaN
  else h = (uint16_t)((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);            // round to nearest, ties to even
  reinterpret_cast<uint16_t*>(row)[v] = h;
}

// grid (rows per sequence, B)
template <int DT>
__global__ __launch_bounds__(kPenaltyThreads) void repetition_penalty_kernel(
    void* z, const int32_t* row_offsets, int rows_per_seq, int n_rows, int V, const int32_t* history, int n_hist,
    const int32_t* x, int k, float theta) {
  const int b = blockIdx.y, i = blockIdx.x, tid = threadIdx.x;
  long row_index = (long)b * rows_per_seq + i;
  if (row_offsets) {                                   // packed rows: sequence b owns [row_offsets[b], row_offsets[b+1])
    const int lo = row_offsets[b], hi = row_offsets[b + 1];
    if (i >= hi - lo || lo < 0 || hi > n_rows) return; // (uniform over the workgroup)
    row_index = (long)lo + i;
  }
  void* row = static_cast<char*>(z) + (size_t)row_index * V * Elem<DT>::bytes;
  const int n_prefix = x ? min(i, k) : 0;
  const int n = n_hist + n_prefix;
  int tok[kPenaltyPerLane];
  float val[kPenaltyPerLane];
#pragma unroll
  for (int j = 0; j < kPenaltyPerLane; ++j) {
    const int idx = tid + j * kPenaltyThreads;
    int t = -1;
    if (idx < n_hist) t = history[(size_t)b * n_hist + idx];
    else if (idx < n) t = x[b * k + (idx - n_hist)];
    if (t < 0 || t >= V) t = -1;                       // padding and impossible ids are ignored
    tok[j] = t;
    val[j] = t >= 0 ? load_elem<DT>(row, t) : 0.f;
  }
  __syncthreads();                                     // every read of this row precedes every write to it
#pragma unroll
  for (int j = 0; j < kPenaltyPerLane; ++j)
    if (tok[j] >= 0) store_elem<DT>(row, tok[j], val[j] < 0.f ? val[j] * theta : val[j] / theta);
}

}  // namespace sv

extern "C" int sv_repetition_penalty(void* z, const int32_t* row_offsets_or_null, int n_rows, int B, int rows_per_seq,
                                     int V, int dtype, const int32_t* history, int n_hist,
                                     const int32_t* x_or_null, int k, float penalty, sv_stream_t stream) {
  using namespace sv;
  SV_REQUIRE(dtype == SV_F32 || dtype == SV_BF16, SV_ERR_DTYPE);
  SV_REQUIRE(B >= 0 && rows_per_seq >= 1 && V >= 1 && n_hist >= 0 && k >= 0, SV_ERR_INVALID_ARG);
  SV_REQUIRE(penalty > 0.f && penalty < INFINITY, SV_ERR_INVALID_ARG);          // (false for NaN)
  SV_REQUIRE(!row_offsets_or_null || n_rows >= 0, SV_ERR_INVALID_ARG);
  SV_REQUIRE(B <= 65535 && rows_per_seq <= 65535 && (long long)n_hist + (x_or_null ? k : 0) <= SV_PENALTY_MAX_TOKENS,
             SV_ERR_TOO_LARGE);
  if (B == 0 || (n_hist == 0 && (!x_or_null || k == 0))) return SV_OK;
  SV_REQUIRE(z && (history || n_hist == 0), SV_ERR_NULL);
  SV_REQUIRE(is_aligned(z, elem_bytes(dtype)) && is_aligned(history, 4) && is_aligned(x_or_null, 4) &&
                 is_aligned(row_offsets_or_null, 4),
             SV_ERR_ALIGN);
  const dim3 grid(rows_per_seq, B), block(kPenaltyThreads);
  hipStream_t st = as_stream(stream);
  if (dtype == SV_F32)
    hipLaunchKernelGGL(repetition_penalty_kernel<DT_F32>, grid, block, 0, st, z, row_offsets_or_null, rows_per_seq,
                       n_rows, V, history, n_hist, x_or_null, k, penalty);
  else
    hipLaunchKernelGGL(repetition_penalty_kernel<DT_BF16>, grid, block, 0, st, z, row_offsets_or_null, rows_per_seq,
                       n_rows, V, history, n_hist, x_or_null, k, penalty);
  return launch_status();
}
