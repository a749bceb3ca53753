// Internal helpers shared by the HIP translation units of libdsbd (not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>
#include "dsbd.h"

#define DSBD_MAX_TREE_NODES 64

#define DSBD_HIP_LAUNCH_CHECK()                      \
  do {                                               \
    hipError_t e__ = hipGetLastError();              \
    if (e__ != hipSuccess) return DSBD_ERR_HIP;      \
  } while (0)

static inline size_t dsbd_align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Carves 256-byte aligned pieces out of a caller-supplied workspace.
struct WorkspaceCarver {
  char* base;
  size_t used;
  explicit WorkspaceCarver(void* p) : base(static_cast<char*>(p)), used(0) {}
  template <typename T>
  T* take(size_t count) {
    used = dsbd_align_up(used, 256);
    T* p = base ? reinterpret_cast<T*>(base + used) : nullptr;
    used += count * sizeof(T);
    return p;
  }
  size_t total() const { return dsbd_align_up(used, 256); }
};

// Measurement hook (timing.hip).  When timing is enabled for `kernel_id`, the launch goes through HIP's extended
// launch call, which stamps a pair of events with the kernel's own start and end on the device (what a profiler's
// kernel trace reports); a pair of hipEventRecord calls around an ordinary launch would also count the dispatch
// latency on either side (2-3 us).  Otherwise an ordinary launch.
bool dsbd_timing_events(int kernel_id, hipEvent_t* start, hipEvent_t* stop);
template <typename F, typename... Args>
inline void dsbd_launch(int kernel_id, F kernel, dim3 grid, dim3 block, unsigned int lds_bytes, hipStream_t stream,
                        Args... args) {
  hipEvent_t e0 = nullptr, e1 = nullptr;
  if (dsbd_timing_events(kernel_id, &e0, &e1))
    hipExtLaunchKernelGGL(kernel, grid, block, lds_bytes, stream, e0, e1, 0, args...);
  else
    hipLaunchKernelGGL(kernel, grid, block, lds_bytes, stream, args...);
}
