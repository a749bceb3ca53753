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

// Tuning overrides and test hooks from the environment, read once per process (knobs.hip).
struct DsbdKnobs {
  int attn_nsplit;             // DSBD_ATTN_NSPLIT: KV splits per (tree, KV head, row block); 0 = the plan's choice
  bool attn_waves8;            // DSBD_ATTN_WAVES8: 8 waves x 16 rows in the shared-tile kernel
  bool attn_staged;            // DSBD_ATTN_STAGED: the register-staged tile kernel also for head size 128
  bool attn_trace;             // DSBD_ATTN_TRACE: timeline of the attention kernel (instrumented builds)
  int stats_chunk;             // DSBD_STATS_CHUNK: logits per workgroup of the statistics pass; 0 = the plan's choice
  int verify_g;                // DSBD_VERIFY_G: workgroups per prompt of the layer kernel; 0 = the plan's choice
  bool verify_trace;           // DSBD_VERIFY_TRACE: timeline of the layer kernel into the workspace ...
  int verify_trace_wg;         // ... of workgroup N - 1 when the variable holds N > 1 (else of the first)
  long long verify_sync_limit_us;   // DSBD_VERIFY_SYNC_LIMIT_US: bound of every wait of the layer kernel; 0 = default
  int verify_mute_wg;          // DSBD_VERIFY_TEST_MUTE_WG: test hook, this workgroup withholds its first post; -1 = none
  int verify_lds_slice;        // DSBD_VERIFY_LDS_SLICE: largest joint slice kept in the LDS; -1 = the plan's choice
  int verify_overlap;          // DSBD_VERIFY_OVERLAP: 0 = statistics pass and layer kernel one after the other
  int warp_fast;               // DSBD_WARP_FAST: 0 = the warping selection always takes its tree form
  int event_fence;             // DSBD_EVENT_FENCE: 1 = the library's cross-stream events keep HIP's system-scope fence; 0 = they order
                               // device work only (no cache write-back for the host's sake at every fork and join)
  int stats_side_lds;          // DSBD_STATS_SIDE_LDS: LDS bytes claimed by a workgroup of the statistics pass when it runs beside
                               // the layer kernel (limits how many of them share a compute unit with it); -1 = the plan's choice
};
const DsbdKnobs& dsbd_knobs();

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
