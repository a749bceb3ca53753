// Forest topology: depth and ancestor-or-self bitmap of every node.
//
// The attention mask of a tree is its topology: a node sees its ancestors and itself
// (paper Section 3.3 and the forest-attention figure).  One 64-thread block per tree, one
// thread per node, each walking its parent chain; the walk validates the parent array so that
// no later kernel ever follows a bad index.
#include "common.h"
#include "topology_device.h"

__global__ __launch_bounds__(64) void topology_kernel(int n_trees, int n_nodes, const int32_t* __restrict__ tree_off,
                                                      const int32_t* __restrict__ parent, int max_tree_nodes,
                                                      int max_depth, int32_t* __restrict__ depth,
                                                      uint64_t* __restrict__ anc_mask, int32_t* __restrict__ fault) {
  const int b = blockIdx.x;
  if (b >= n_trees) return;
  const int bad = dsbd_tree_topology(b, threadIdx.x, n_nodes, tree_off, parent, max_tree_nodes, max_depth, depth, anc_mask);
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
