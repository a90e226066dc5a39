// The bench-only library (libftar_measure.so): the C entry point of the bare streaming kernels
// declared in include/ftar_measure.h.  Links against libftar.so, whose launch path (tuning
// overrides, dispatch-recorded timing events) the probe kernels share.

#include <cstring>

#include "ftar_internal.h"
#include "ftar_measure.h"

using namespace ftar;

extern "C" {

ftar_status_t ftar_probe_stream(void* const* bufs, int n_read, int n_written, size_t bytes, uint32_t fill,
                                void* stream) {
  if (!bufs || n_read < 0 || n_written < 0 || n_read + n_written < 1 || n_read + n_written > kMaxReplicas ||
      bytes == 0 || bytes % (32 * 1024) != 0)
    return FTAR_ERR_INVALID_ARG;
  PtrTable tab;
  std::memset(&tab, 0, sizeof(tab));
  for (int j = 0; j < n_read + n_written; ++j) {
    if (!bufs[j] || reinterpret_cast<uintptr_t>(bufs[j]) % 16 != 0) return FTAR_ERR_INVALID_ARG;
    tab.p[j] = bufs[j];
  }
  hipError_t e = launch_probe_stream(tab, n_read, n_written, bytes / 16, fill, static_cast<hipStream_t>(stream));
  if (e == hipErrorInvalidValue) return FTAR_ERR_INVALID_ARG;
  return e == hipSuccess ? FTAR_OK : FTAR_ERR_DEVICE;
}

ftar_status_t ftar_probe_stream_windows(void* const* bufs, int n_read, size_t bytes, unsigned period_ticks,
                                        unsigned window_ticks, void* stream) {
  if (!bufs || n_read < 1 || n_read + 1 > kMaxReplicas || bytes == 0 || bytes % (32 * 1024) != 0 ||
      period_ticks < 2 || (period_ticks & (period_ticks - 1)) != 0 || window_ticks == 0 || window_ticks > period_ticks)
    return FTAR_ERR_INVALID_ARG;
  PtrTable tab;
  std::memset(&tab, 0, sizeof(tab));
  for (int j = 0; j < n_read + 1; ++j) {
    if (!bufs[j] || reinterpret_cast<uintptr_t>(bufs[j]) % 16 != 0) return FTAR_ERR_INVALID_ARG;
    tab.p[j] = bufs[j];
  }
  hipError_t e = launch_probe_stream_win(tab, n_read, bytes / 16, period_ticks, window_ticks,
                                         static_cast<hipStream_t>(stream));
  if (e == hipErrorInvalidValue) return FTAR_ERR_INVALID_ARG;
  return e == hipSuccess ? FTAR_OK : FTAR_ERR_DEVICE;
}

ftar_status_t ftar_probe_stream_workgroups(void* const* bufs, int n_read, size_t bytes, unsigned n_workgroups,
                                           unsigned threads, unsigned vectors_per_lane, void* stream) {
  if (!bufs || n_read < 1 || n_read > 2 || bytes == 0 || n_workgroups == 0 || n_workgroups > 4096 || threads == 0 ||
      vectors_per_lane == 0 || bytes % (static_cast<size_t>(threads) * vectors_per_lane * 16) != 0)
    return FTAR_ERR_INVALID_ARG;
  PtrTable tab;
  std::memset(&tab, 0, sizeof(tab));
  for (int j = 0; j < n_read + 1; ++j) {
    if (!bufs[j] || reinterpret_cast<uintptr_t>(bufs[j]) % 16 != 0) return FTAR_ERR_INVALID_ARG;
    tab.p[j] = bufs[j];
  }
  hipError_t e = launch_probe_few(tab, n_read, bytes / 16, n_workgroups, threads, vectors_per_lane,
                                  static_cast<hipStream_t>(stream));
  if (e == hipErrorInvalidValue) return FTAR_ERR_INVALID_ARG;
  return e == hipSuccess ? FTAR_OK : FTAR_ERR_DEVICE;
}

}  // extern "C"
