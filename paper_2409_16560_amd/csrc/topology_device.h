// Forest topology of one tree, computed by one 64-lane wave (paper Section 3.3 and the forest-attention figure:
// a node sees its ancestors and itself, so the attention mask of a tree is its topology).
#pragma once
#include "common.h"

// Node range of tree b as the kernels use it: n_all nodes in the forest arrays, of which the first n are followed.
struct dsbd_tree_range {
  int base, n_all, n;
  int bad;          // DSBD_FAULT_* bits found so far (uniform over the wave)
  bool valid;       // false: the offsets are unusable and nothing of the tree may be touched
};

__device__ __forceinline__ dsbd_tree_range dsbd_tree_range_of(int b, int n_nodes, const int32_t* __restrict__ tree_off,
                                                              int max_tree_nodes) {
  dsbd_tree_range t;
  t.base = tree_off[b];
  const int end = tree_off[b + 1];
  t.bad = 0;
  t.valid = !(t.base < 0 || end > n_nodes || end <= t.base);
  t.n_all = t.valid ? end - t.base : 0;
  t.n = t.n_all;
  if (!t.valid) t.bad |= DSBD_FAULT_TOPOLOGY;
  if (t.n > max_tree_nodes || t.n > DSBD_MAX_TREE_NODES) {
    t.bad |= DSBD_FAULT_BOUNDS;
    t.n = min(t.n, min(max_tree_nodes, DSBD_MAX_TREE_NODES));
  }
  return t;
}

// This lane's entry of the tree's parent array (global index of node `lane`'s parent; -1 beyond the tree).
__device__ __forceinline__ int dsbd_tree_parent_of(const dsbd_tree_range& t, int lane, const int32_t* __restrict__ parent) {
  return (t.valid && lane < t.n) ? parent[t.base + lane] : -1;
}

// Lane j handles node j: every lane walks its node's parent chain through lane shuffles of the entries loaded by
// dsbd_tree_parent_of, validating them on the way, so the walk costs no further memory round trips.  Writes the
// node's depth and ancestor-or-self bitmap (either output may be null; *m_out, if given, receives this lane's
// bitmap, 0 beyond the tree) and returns the DSBD_FAULT_* bits this lane found (those of the range included, in
// lane 0).  Must be called by all 64 lanes of a wave; nothing is read or written outside the tree's node range.
__device__ __forceinline__ int dsbd_tree_walk(const dsbd_tree_range& t, int lane, int p_mine, int max_depth,
                                              int32_t* __restrict__ depth, uint64_t* __restrict__ anc_mask,
                                              uint64_t* m_out) {
  if (m_out) *m_out = 0;
  int bad = lane == 0 ? t.bad : 0;
  if (!t.valid) return bad;
  const int base = t.base, n = t.n;
  // nodes beyond the supported tree size: defined (empty) outputs, never followed
  for (int j = n + lane; j < t.n_all; j += 64) {
    if (anc_mask) anc_mask[base + j] = 0;
    if (depth) depth[base + j] = 0;
  }
  const int j = lane;
  uint64_t m = 0;
  int a = j;                        // local index of the node the walk stands on
  bool ok = true;
  bool done = !(j < n);
  for (int it = 0; it < DSBD_MAX_TREE_NODES; ++it) {
    if (!done) m |= 1ull << a;
    const int p = __shfl(p_mine, a);                  // every lane takes part; a is always a lane of the tree
    if (!done) {
      if (a == 0) {
        if (p != -1) ok = false;                      // the first node of a tree is its root
        done = true;
      } else {
        const int pl = p - base;
        if (pl < 0 || pl >= a) { ok = false; done = true; }   // outside the tree, or not before the child
        else a = pl;
      }
    }
    if (__ballot(!done) == 0ull) break;
  }
  if (j < n) {
    if (!ok) {
      bad |= DSBD_FAULT_TOPOLOGY;
      m = 1ull << j;                // fall back to "sees only itself"
    }
    const int d = __popcll(m) - 1;
    if (d > max_depth) bad |= DSBD_FAULT_BOUNDS;
    if (anc_mask) anc_mask[base + j] = m;
    if (depth) depth[base + j] = d;
    if (m_out) *m_out = m;
  }
  return bad;
}

__device__ __forceinline__ int dsbd_tree_topology(int b, int lane, int n_nodes, const int32_t* __restrict__ tree_off,
                                                  const int32_t* __restrict__ parent, int max_tree_nodes, int max_depth,
                                                  int32_t* __restrict__ depth, uint64_t* __restrict__ anc_mask,
                                                  uint64_t* m_out) {
  const dsbd_tree_range t = dsbd_tree_range_of(b, n_nodes, tree_off, max_tree_nodes);
  return dsbd_tree_walk(t, lane, dsbd_tree_parent_of(t, lane, parent), max_depth, depth, anc_mask, m_out);
}
