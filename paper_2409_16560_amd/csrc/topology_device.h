// Forest topology of one tree, computed by one 64-lane wave (paper Section 3.3 and the forest-attention figure:
// a node sees its ancestors and itself, so the attention mask of a tree is its topology).
#pragma once
#include "common.h"

// Lane j handles node j of tree b: walks its parent chain, validating the parent array on the way, and writes
// the node's depth and ancestor-or-self bitmap (either output may be null).  Returns the DSBD_FAULT_* bits this
// lane found; nothing is ever read or written outside the tree's node range.
__device__ __forceinline__ int dsbd_tree_topology(int b, int lane, int n_nodes, const int32_t* __restrict__ tree_off,
                                                  const int32_t* __restrict__ parent, int max_tree_nodes, int max_depth,
                                                  int32_t* __restrict__ depth, uint64_t* __restrict__ anc_mask) {
  const int base = tree_off[b];
  const int end = tree_off[b + 1];
  if (base < 0 || end > n_nodes || end <= base) return lane == 0 ? DSBD_FAULT_TOPOLOGY : 0;
  int bad = 0;
  const int n_all = end - base;
  int n = n_all;
  if (n > max_tree_nodes || n > DSBD_MAX_TREE_NODES) {
    bad |= DSBD_FAULT_BOUNDS;
    n = min(n, min(max_tree_nodes, DSBD_MAX_TREE_NODES));
  }
  // nodes beyond the supported tree size: defined (empty) outputs, never followed
  for (int j = n + lane; j < n_all; j += 64) {
    if (anc_mask) anc_mask[base + j] = 0;
    if (depth) depth[base + j] = 0;
  }
  const int j = lane;
  if (j < n) {
    uint64_t m = 0;
    int a = j;                      // local index
    bool ok = true;
    for (int it = 0; it < DSBD_MAX_TREE_NODES; ++it) {
      m |= 1ull << a;
      const int p = parent[base + a];
      if (a == 0) {
        if (p != -1) ok = false;
        break;
      }
      const int pl = p - base;
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
    const int d = __popcll(m) - 1;
    if (d > max_depth) bad |= DSBD_FAULT_BOUNDS;
    if (anc_mask) anc_mask[base + j] = m;
    if (depth) depth[base + j] = d;
  }
  return bad;
}
