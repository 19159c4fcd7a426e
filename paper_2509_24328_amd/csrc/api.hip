// Shape-independent parts of the C ABI: status strings and workspace sizing.
#include <atomic>
#include <mutex>

#include "sv_device.hpp"
#include "sv_host.hpp"

extern "C" const char* sv_strerror(int status) {
  switch (status) {
    case SV_OK: return "SV_OK";
    case SV_ERR_INVALID_ARG: return "SV_ERR_INVALID_ARG: a size is out of range or inconsistent";
    case SV_ERR_NULL: return "SV_ERR_NULL: a required pointer is NULL";
    case SV_ERR_DTYPE: return "SV_ERR_DTYPE: dtype is neither SV_F32 nor SV_BF16";
    case SV_ERR_ALIGN: return "SV_ERR_ALIGN: a pointer is not aligned to its element type";
    case SV_ERR_WORKSPACE: return "SV_ERR_WORKSPACE: workspace is NULL, misaligned or too small";
    case SV_ERR_LAUNCH: return "SV_ERR_LAUNCH: the HIP runtime rejected a kernel launch";
    case SV_ERR_TOO_LARGE: return "SV_ERR_TOO_LARGE: problem exceeds a documented library limit";
    default: return "unknown sv status";
  }
}

extern "C" size_t sv_workspace_bytes(int B, int k, int V, int dtype) {
  if (B < 0 || k < 1 || V < 1 || sv::elem_bytes(dtype) == 0) return 0;
  if (B == 0) return sv::kWsAlign;
  return sv::carve_verify_ws(nullptr, B, k, V).bytes;
}

namespace sv {
namespace {
TimingTap g_taps[SV_KERNEL_COUNT] = {};
std::mutex g_taps_mutex;
std::atomic<int> g_taps_set{0};      // number of kernels with a pair set: launches skip the lock while it is 0
}  // namespace

TimingTap timing_tap(int kernel) {
  if (g_taps_set.load(std::memory_order_acquire) == 0) return TimingTap{nullptr, nullptr};
  std::lock_guard<std::mutex> lock(g_taps_mutex);
  return g_taps[kernel];             // both handles of one setting, never half of each
}
}  // namespace sv

extern "C" int sv_set_timing_events(int kernel, void* start_event, void* stop_event) {
  if (kernel < 0 || kernel >= SV_KERNEL_COUNT) return SV_ERR_INVALID_ARG;
  if ((start_event == nullptr) != (stop_event == nullptr)) return SV_ERR_INVALID_ARG;
  std::lock_guard<std::mutex> lock(sv::g_taps_mutex);
  const bool was = sv::g_taps[kernel].start != nullptr, is = start_event != nullptr;
  sv::g_taps[kernel].start = reinterpret_cast<hipEvent_t>(start_event);
  sv::g_taps[kernel].stop = reinterpret_cast<hipEvent_t>(stop_event);
  sv::g_taps_set.fetch_add((is ? 1 : 0) - (was ? 1 : 0), std::memory_order_release);
  return SV_OK;
}

namespace sv {
// one lane per (sequence, position): both uniforms of its counter
__global__ void uniforms_kernel(uint32_t seed_lo, uint32_t seed_hi, uint32_t step, int B, int n_pos,
                                double* u_accept, double* u_sample) {
  const long j = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (j >= (long)B * n_pos) return;
  const uint32_t b = (uint32_t)(j / n_pos), i = (uint32_t)(j % n_pos);
  const U4 r = philox4x32_10(i, b, 0u, step, seed_lo, seed_hi);
  u_accept[j] = unit_from_word(r.w[0]);
  u_sample[j] = unit_from_word(r.w[1]);
}
}  // namespace sv

extern "C" int sv_uniforms(uint64_t seed, uint32_t step, int B, int n_pos, double* u_accept, double* u_sample,
                           sv_stream_t stream) {
  using namespace sv;
  SV_REQUIRE(B >= 0 && n_pos >= 1, SV_ERR_INVALID_ARG);
  SV_REQUIRE((long long)B * n_pos <= 0x7fffffffLL, SV_ERR_TOO_LARGE);
  if (B == 0) return SV_OK;
  SV_REQUIRE(u_accept && u_sample, SV_ERR_NULL);
  SV_REQUIRE(is_aligned(u_accept, 8) && is_aligned(u_sample, 8), SV_ERR_ALIGN);
  const long n = (long)B * n_pos;
  hipLaunchKernelGGL(uniforms_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, as_stream(stream),
                     (uint32_t)(seed & 0xffffffffu), (uint32_t)(seed >> 32), step, B, n_pos, u_accept, u_sample);
  return launch_status();
}
