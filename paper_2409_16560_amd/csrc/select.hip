// Next beam set from the verification outputs (paper Algorithm 1, return statement; Section 3.3 last
// paragraph: the caches kept are those the output beams descend from; Section 3.4: the memory-reduced
// variant keeps only the output beam of lowest perplexity).
//
// One 64-thread block per prompt; one thread per output beam walks from the beam's parent node up to
// its root and writes the path root-first.  All output beams of a prompt have the same length, so the
// lowest perplexity is the highest cumulative target log-likelihood (ties: lowest output index).
#include "common.h"

#define SELECT_LDS_TREES 8192

struct SelectArgs {
  int n_prompts, n_trees, n_nodes, W_cap, Lmax, keep_one;
  int toff_in_lds;       // tree_off staged in the dynamic LDS (forests of up to SELECT_LDS_TREES trees), else read in place
  const int32_t *tree_off, *parent;
  const int32_t *n_out, *out_parent, *out_token;
  const double *out_lp, *out_lq;
  dsbd_next_beams nx;
  int32_t* fault;
};

__global__ __launch_bounds__(64) void select_beams_kernel(SelectArgs a) {
  const int p = blockIdx.x;
  const int j = threadIdx.x;
  const int W = a.W_cap;
  const int plen = a.Lmax + 1;
  int n = a.n_out[p];
  n = max(0, min(n, min(W, 64)));
  __shared__ int best;
  __shared__ int path_lds[64][DSBD_MAX_TREE_NODES + 1];   // one row per output beam (padded against bank conflicts)
  extern __shared__ int toff_lds[];                       // tree_off[0 .. n_trees], staged once for the searches
  if (a.toff_in_lds)
    for (int t = j; t <= a.n_trees; t += 64) toff_lds[t] = a.tree_off[t];
  const int* const toff = a.toff_in_lds ? toff_lds : a.tree_off;
  if (j == 0) {
    best = 0;
    if (a.keep_one)
      for (int k = 1; k < n; ++k)
        if (a.out_lp[(long long)p * W + k] > a.out_lp[(long long)p * W + best]) best = k;
    a.nx.n_next[p] = a.keep_one ? min(n, 1) : n;
  }
  __syncthreads();
  const int n_next = a.keep_one ? min(n, 1) : n;
  if (j >= W) return;
  const long long o = (long long)p * W + j;
  int32_t* path = a.nx.path + o * plen;
  if (j >= n_next) {
    a.nx.src_tree[o] = -1; a.nx.src_out[o] = -1; a.nx.path_len[o] = 0; a.nx.token[o] = -1;
    a.nx.logp_target[o] = 0.0; a.nx.logp_draft[o] = 0.0;
    for (int k = 0; k < plen; ++k) path[k] = -1;
    return;
  }
  const int src = a.keep_one ? best : j;
  const long long so = (long long)p * W + src;
  int node = a.out_parent[so];
  int len = 0, bad = 0;
  int* tmp = path_lds[j];
  int root = -1;
  if (node < 0 || node >= a.n_nodes) { bad = DSBD_FAULT_TOPOLOGY; }
  else {
    int cur = node;
    for (int it = 0; it < DSBD_MAX_TREE_NODES; ++it) {
      tmp[len++] = cur;
      const int par = a.parent[cur];
      if (par < 0) { root = cur; break; }
      if (par >= cur) { bad = DSBD_FAULT_TOPOLOGY; break; }
      cur = par;
    }
    if (root < 0) bad = DSBD_FAULT_TOPOLOGY;
    if (len > plen) { bad |= DSBD_FAULT_BOUNDS; }
  }
  if (bad) { atomicOr(a.fault, bad); len = 0; root = -1; }
  // tree of the root by binary search in tree_off
  int tree = -1;
  if (root >= 0) {
    int lo = 0, hi = a.n_trees;
    while (lo < hi) { const int mid = (lo + hi) >> 1; if (toff[mid + 1] <= root) lo = mid + 1; else hi = mid; }
    tree = lo < a.n_trees ? lo : -1;
  }
  a.nx.src_tree[o] = tree;
  a.nx.src_out[o] = src;
  a.nx.path_len[o] = len;
  for (int k = 0; k < plen; ++k) path[k] = k < len ? tmp[len - 1 - k] : -1;
  a.nx.token[o] = a.out_token[so];
  a.nx.logp_target[o] = a.out_lp[so];
  a.nx.logp_draft[o] = a.out_lq[so];
}

extern "C" int32_t dsbd_select_beams(const dsbd_forest* f, const dsbd_verify_out* v, int32_t W_cap, int32_t keep_one,
                                     const dsbd_next_beams* nx, int32_t* fault, void* stream_) {
  if (!f || !v || !nx || !fault) return DSBD_ERR_INVALID;
  if (W_cap < 1 || W_cap > 64) return DSBD_ERR_UNSUPPORTED;
  if (f->max_depth < 0 || f->max_depth >= DSBD_MAX_TREE_NODES) return DSBD_ERR_INVALID;
  if (f->n_prompts == 0) return DSBD_OK;
  if (f->n_prompts < 0 || !f->tree_off || !f->parent) return DSBD_ERR_INVALID;
  if (!v->n_out || !v->out_parent || !v->out_token || !v->out_logp_target || !v->out_logp_draft)
    return DSBD_ERR_INVALID;
  if (!nx->n_next || !nx->src_tree || !nx->src_out || !nx->path_len || !nx->path || !nx->token || !nx->logp_target ||
      !nx->logp_draft)
    return DSBD_ERR_INVALID;
  SelectArgs a;
  a.n_prompts = f->n_prompts; a.n_trees = f->n_trees; a.n_nodes = f->n_nodes; a.W_cap = W_cap;
  a.Lmax = f->max_depth; a.keep_one = keep_one != 0;
  a.tree_off = f->tree_off; a.parent = f->parent;
  a.n_out = v->n_out; a.out_parent = v->out_parent; a.out_token = v->out_token;
  a.out_lp = v->out_logp_target; a.out_lq = v->out_logp_draft;
  a.nx = *nx; a.fault = fault;
  // static (16.6 KB) + dynamic LDS must stay within the 64 KB a launch gets without asking for more: larger forests
  // search tree_off where it lies
  size_t toff_bytes = ((size_t)f->n_trees + 1) * sizeof(int32_t);
  a.toff_in_lds = toff_bytes <= SELECT_LDS_TREES * sizeof(int32_t) ? 1 : 0;
  if (!a.toff_in_lds) toff_bytes = 0;
  hipLaunchKernelGGL(select_beams_kernel, dim3(f->n_prompts), dim3(64), toff_bytes, static_cast<hipStream_t>(stream_), a);
  DSBD_HIP_LAUNCH_CHECK();
  return DSBD_OK;
}

extern "C" const char* dsbd_version(void) { return "dsbd 0.6 (gfx950)"; }
