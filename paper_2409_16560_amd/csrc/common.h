// Internal helpers shared by the HIP translation units of libdsbd (not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
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

// Measurement hook (timing.hip): records an event before / after kernel `kernel_id` when enabled.
void dsbd_timing_mark(int kernel_id, bool begin, hipStream_t stream);
