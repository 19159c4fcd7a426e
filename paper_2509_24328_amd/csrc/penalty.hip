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

// The tensors of one launch (draft, companion and target logits of a step share the history).
struct PenaltyBatch {
  int n;
  void* z[SV_WARP_MAX_TENSORS];
  const int32_t* row_offsets[SV_WARP_MAX_TENSORS];   // nullable: packed rows
  int n_rows[SV_WARP_MAX_TENSORS];
  int rows_per_seq[SV_WARP_MAX_TENSORS];
};

// grid (rows per sequence, B, tensors)
template <int DT>
__global__ __launch_bounds__(kPenaltyThreads) void repetition_penalty_kernel(
    PenaltyBatch pb, int V, const int32_t* history, int n_hist, const int32_t* x, int k, float theta) {
  const int t = blockIdx.z, b = blockIdx.y, i = blockIdx.x, tid = threadIdx.x;
  if (i >= pb.rows_per_seq[t]) return;                 // (uniform over the workgroup)
  long row_index = (long)b * pb.rows_per_seq[t] + i;
  if (const int32_t* row_offsets = pb.row_offsets[t]) {   // packed rows: sequence b owns [row_offsets[b], row_offsets[b+1])
    const int lo = row_offsets[b], hi = row_offsets[b + 1];
    if (i >= hi - lo || lo < 0 || hi > pb.n_rows[t]) return;
    row_index = (long)lo + i;
  }
  void* row = static_cast<char*>(pb.z[t]) + (size_t)row_index * V * Elem<DT>::bytes;
  const int n_prefix = x ? min(i, k) : 0;
  const int n = n_hist + n_prefix;
  int tok[kPenaltyPerLane];
  float val[kPenaltyPerLane];
#pragma unroll
  for (int j = 0; j < kPenaltyPerLane; ++j) {
    const int idx = tid + j * kPenaltyThreads;
    int tk = -1;
    if (idx < n_hist) tk = history[(size_t)b * n_hist + idx];
    else if (idx < n) tk = x[b * k + (idx - n_hist)];
    if (tk < 0 || tk >= V) tk = -1;                    // padding and impossible ids are ignored
    tok[j] = tk;
    val[j] = tk >= 0 ? load_elem<DT>(row, tk) : 0.f;
  }
  __syncthreads();                                     // every read of this row precedes every write to it
#pragma unroll
  for (int j = 0; j < kPenaltyPerLane; ++j)
    if (tok[j] >= 0) store_elem<DT>(row, tok[j], val[j] < 0.f ? val[j] * theta : val[j] / theta);
}

}  // namespace sv

namespace {
int launch_penalty(int n, void* const* z, const int32_t* const* row_offsets, const int* n_rows, int B,
                   const int* rows_per_seq, int V, int dtype, const int32_t* history, int n_hist,
                   const int32_t* x, int k, float penalty, sv_stream_t stream) {
  using namespace sv;
  SV_REQUIRE(dtype == SV_F32 || dtype == SV_BF16, SV_ERR_DTYPE);
  SV_REQUIRE(n >= 1 && n <= SV_WARP_MAX_TENSORS && B >= 0 && V >= 1 && n_hist >= 0 && k >= 0, SV_ERR_INVALID_ARG);
  SV_REQUIRE(penalty > 0.f && penalty < INFINITY, SV_ERR_INVALID_ARG);          // (false for NaN)
  SV_REQUIRE(B <= 65535 && (long long)n_hist + (x ? k : 0) <= SV_PENALTY_MAX_TOKENS, SV_ERR_TOO_LARGE);
  PenaltyBatch pb = {};
  pb.n = n;
  int max_rows = 0;
  for (int t = 0; t < n; ++t) {
    SV_REQUIRE(rows_per_seq[t] >= 1 && (!row_offsets || !row_offsets[t] || n_rows[t] >= 0), SV_ERR_INVALID_ARG);
    SV_REQUIRE(rows_per_seq[t] <= 65535, SV_ERR_TOO_LARGE);
    max_rows = rows_per_seq[t] > max_rows ? rows_per_seq[t] : max_rows;
  }
  if (B == 0 || (n_hist == 0 && (!x || k == 0))) return SV_OK;
  SV_REQUIRE(history || n_hist == 0, SV_ERR_NULL);
  SV_REQUIRE(is_aligned(history, 4) && is_aligned(x, 4), SV_ERR_ALIGN);
  for (int t = 0; t < n; ++t) {
    SV_REQUIRE(z[t], SV_ERR_NULL);
    pb.z[t] = z[t];
    pb.row_offsets[t] = row_offsets ? row_offsets[t] : nullptr;
    pb.n_rows[t] = n_rows ? n_rows[t] : 0;
    pb.rows_per_seq[t] = rows_per_seq[t];
    SV_REQUIRE(is_aligned(z[t], elem_bytes(dtype)) && is_aligned(pb.row_offsets[t], 4), SV_ERR_ALIGN);
  }
  const dim3 grid(max_rows, B, n), block(kPenaltyThreads);
  hipStream_t st = as_stream(stream);
  if (dtype == SV_F32)
    hipLaunchKernelGGL(repetition_penalty_kernel<DT_F32>, grid, block, 0, st, pb, V, history, n_hist, x, k, penalty);
  else
    hipLaunchKernelGGL(repetition_penalty_kernel<DT_BF16>, grid, block, 0, st, pb, V, history, n_hist, x, k, penalty);
  return launch_status();
}
}  // namespace

extern "C" int sv_repetition_penalty(void* z, const int32_t* row_offsets_or_null, int n_rows, int B, int rows_per_seq,
                                     int V, int dtype, const int32_t* history, int n_hist,
                                     const int32_t* x_or_null, int k, float penalty, sv_stream_t stream) {
  return launch_penalty(1, &z, &row_offsets_or_null, &n_rows, B, &rows_per_seq, V, dtype, history, n_hist, x_or_null, k,
                        penalty, stream);
}

extern "C" int sv_repetition_penalty_multi(int n, void* const* z, const int32_t* const* row_offsets_or_null,
                                           const int* n_rows_or_null, int B, const int* rows_per_seq, int V, int dtype,
                                           const int32_t* history, int n_hist, const int32_t* x_or_null, int k,
                                           float penalty, sv_stream_t stream) {
  SV_REQUIRE(n >= 1 && n <= SV_WARP_MAX_TENSORS, SV_ERR_INVALID_ARG);
  SV_REQUIRE(z && rows_per_seq && (!row_offsets_or_null || n_rows_or_null), SV_ERR_NULL);
  return launch_penalty(n, z, row_offsets_or_null, n_rows_or_null, B, rows_per_seq, V, dtype, history, n_hist,
                        x_or_null, k, penalty, stream);
}
