// Shape-independent parts of the C ABI: status strings and workspace sizing.
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
TimingTap g_taps[SV_KERNEL_COUNT] = {};
}

extern "C" int sv_set_timing_events(int kernel, void* start_event, void* stop_event) {
  if (kernel < 0 || kernel >= SV_KERNEL_COUNT) return SV_ERR_INVALID_ARG;
  if ((start_event == nullptr) != (stop_event == nullptr)) return SV_ERR_INVALID_ARG;
  sv::g_taps[kernel].start = reinterpret_cast<hipEvent_t>(start_event);
  sv::g_taps[kernel].stop = reinterpret_cast<hipEvent_t>(stop_event);
  return SV_OK;
}
