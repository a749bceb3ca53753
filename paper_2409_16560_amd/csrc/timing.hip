// Measurement hook: HIP events stamped with the start and end of ONE chosen kernel, on the stream that kernel is
// launched on (extended launch call, see dsbd_launch), so a benchmark can read that kernel's duration per call
// without a profiler attached.  Off by default; the only state the library keeps.
#include "common.h"
#include <vector>

namespace {
int g_kernel = 0;
std::vector<hipEvent_t> g_start, g_stop;
size_t g_used = 0;
}  // namespace

bool dsbd_timing_events(int kernel_id, hipEvent_t* start, hipEvent_t* stop) {
  if (kernel_id != g_kernel || g_kernel == 0 || g_used >= g_start.size()) return false;
  *start = g_start[g_used]; *stop = g_stop[g_used];
  ++g_used;
  return true;
}

extern "C" int32_t dsbd_timing_enable(int32_t kernel_id, int32_t capacity) {
  for (hipEvent_t e : g_start) (void)hipEventDestroy(e);
  for (hipEvent_t e : g_stop) (void)hipEventDestroy(e);
  g_start.clear(); g_stop.clear(); g_used = 0; g_kernel = 0;
  if (kernel_id == 0) return DSBD_OK;
  if (kernel_id < 0 || kernel_id > DSBD_KERNEL_KV_COMMIT || capacity < 1) return DSBD_ERR_INVALID;
  for (int i = 0; i < capacity; ++i) {
    hipEvent_t a, b;
    if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) return DSBD_ERR_HIP;
    g_start.push_back(a); g_stop.push_back(b);
  }
  g_kernel = kernel_id;
  return DSBD_OK;
}

extern "C" int32_t dsbd_timing_collect(float* ms, int32_t max_n) {
  int n = 0;
  for (size_t i = 0; i < g_used && n < max_n; ++i) {
    if (hipEventSynchronize(g_stop[i]) != hipSuccess) return DSBD_ERR_HIP;
    float t = 0.f;
    if (hipEventElapsedTime(&t, g_start[i], g_stop[i]) != hipSuccess) return DSBD_ERR_HIP;
    ms[n++] = t;
  }
  g_used = 0;
  return n;
}
