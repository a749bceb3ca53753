// Forest topology: depth and ancestor-or-self bitmap of every node.
//
// The attention mask of a tree is its topology: a node sees its ancestors and itself
// (paper Section 3.3 and the forest-attention figure).  One 64-thread block per tree, one
// thread per node, each walking its parent chain; the walk validates the parent array so that
// no later kernel ever follows a bad index.
#include "common.h"

__global__ __launch_bounds__(64) void topology_kernel(int n_trees, int n_nodes, const int32_t* __restrict__ tree_off,
                                                      const int32_t* __restrict__ parent, int max_tree_nodes,
                                                      int max_depth, int32_t* __restrict__ depth,
                                                      uint64_t* __restrict__ anc_mask, int32_t* __restrict__ fault) {
  const int b = blockIdx.x;
  if (b >= n_trees) return;
  int base = tree_off[b];
  int end = tree_off[b + 1];
  int bad = 0;
  if (base < 0 || end > n_nodes || end <= base) {
    if (threadIdx.x == 0) atomicOr(fault, DSBD_FAULT_TOPOLOGY);
    return;
  }
  const int n_all = end - base;
  int n = n_all;
  if (n > max_tree_nodes || n > DSBD_MAX_TREE_NODES) {
    bad |= DSBD_FAULT_BOUNDS;
    n = min(n, min(max_tree_nodes, DSBD_MAX_TREE_NODES));
  }
  // nodes beyond the supported tree size: defined (empty) outputs, never followed
  for (int j = n + threadIdx.x; j < n_all; j += blockDim.x) {
    anc_mask[base + j] = 0;
    if (depth) depth[base + j] = 0;
  }
  const int j = threadIdx.x;
  if (j < n) {
    uint64_t m = 0;
    int a = j;                      // local index
    bool ok = true;
    for (int it = 0; it < DSBD_MAX_TREE_NODES; ++it) {
      m |= 1ull << a;
      int p = parent[base + a];
      if (a == 0) {
        if (p != -1) ok = false;
        break;
      }
      int pl = p - base;
      if (pl < 0 || pl >= a) {      // outside the tree, or not before the child
        ok = false;
        break;
      }
      a = pl;
    }
    if (!ok) {
      bad |= DSBD_FAULT_TOPOLOGY;
      m = 1ull << j;                // fall back to "sees only itself"
    }
    int d = __popcll(m) - 1;
    if (d > max_depth) bad |= DSBD_FAULT_BOUNDS;
    anc_mask[base + j] = m;
    if (depth) depth[base + j] = d;
  }
  if (bad) atomicOr(fault, bad);
}

int32_t dsbd_launch_topology(const dsbd_forest* f, int32_t* depth, uint64_t* anc_mask, int32_t* fault,
                             hipStream_t stream) {
  if (f->n_nodes > 0) {
    hipLaunchKernelGGL(topology_kernel, dim3(f->n_trees), dim3(64), 0, stream, f->n_trees, f->n_nodes, f->tree_off,
                       f->parent, f->max_tree_nodes, f->max_depth, depth, anc_mask, fault);
    DSBD_HIP_LAUNCH_CHECK();
  }
  return DSBD_OK;
}
