// Draft stage (Section 3.1 "Overview" / "Details"): one beam-sampling step of the small model, and the layout of
// the sampled layers as a draft forest.
//
// dsbd_draft_layer: W_S independent draws from q_beam = T o q/Q over (beams of the current layer) x V are what
// the verification's additional layer does with p_beam: the call presents the layer's beams as a forest of
// single-node trees (no draft layers), the small model's logits as both models', and runs the verification
// kernels; their "additional layer" then is the W_S draws.
//
// dsbd_build_forest: one workgroup per prompt turns the layers' (parent row, token) lists into the
// tree-contiguous layout the other calls expect.
#include "common.h"

#define DR_BLOCK 256
#define BF_BLOCK 512
#define BF_NODE_CAP 512

namespace {

struct DraftSetupArgs {
  int n_prompts, n_beams, W_S;
  const int32_t* beam_off;
  const float* u;
  int32_t *tree_prompt, *tree_off, *parent, *token;
  float *u_accept, *u_resid, *u_fill;
  int32_t* fault;
};

// beams as single-node trees; uniforms into the layout of the verification (row 1 = its additional layer)
__global__ __launch_bounds__(DR_BLOCK) void draft_setup_kernel(DraftSetupArgs a) {
  const long long i = (long long)blockIdx.x * DR_BLOCK + threadIdx.x;
  if (i == 0 && (a.beam_off[0] != 0 || a.beam_off[a.n_prompts] != a.n_beams)) atomicOr(a.fault, DSBD_FAULT_TOPOLOGY);
  if (i < a.n_beams) {
    // prompt of beam i: the last p with beam_off[p] <= i
    int lo = 0, hi = a.n_prompts - 1;
    while (lo < hi) {
      const int mid = (lo + hi + 1) >> 1;
      if (a.beam_off[mid] <= i) lo = mid; else hi = mid - 1;
    }
    a.tree_prompt[i] = lo;
    a.tree_off[i] = (int)i;
    a.parent[i] = -1;
    a.token[i] = 0;
    a.u_accept[i] = 0.f;
  }
  if (i == a.n_beams) a.tree_off[i] = a.n_beams;
  if (i < 2LL * a.n_prompts) a.u_resid[i] = 0.f;
  if (i < 2LL * a.n_prompts * a.W_S) {
    const int p = (int)(i / (2 * a.W_S)), rest = (int)(i % (2 * a.W_S));
    a.u_fill[i] = rest >= a.W_S ? a.u[(long long)p * a.W_S + rest - a.W_S] : 0.f;
  }
}

struct DraftScratch {
  int32_t *tree_prompt, *tree_off, *parent, *token;
  float *u_accept, *u_resid, *u_fill;
  uint8_t* node_status;
  int32_t *l_last, *layer_width, *n_out, *out_node, *near_tie;
  double* out_logp_other;
  void* verify_ws;
};

void make_forest(const dsbd_draft_in* in, const DraftScratch& s, dsbd_forest* f) {
  f->n_prompts = in->n_prompts; f->n_trees = in->n_beams; f->n_nodes = in->n_beams;
  f->tree_prompt = s.tree_prompt; f->tree_off = s.tree_off; f->parent = s.parent; f->token = s.token;
  f->draft_rank = nullptr;
  f->max_tree_nodes = 1; f->max_depth = 0; f->max_prompt_trees = in->max_prompt_beams;
}

dsbd_params make_params(int32_t W_S, int32_t top_k, float top_p) {
  dsbd_params p;
  p.W_L = W_S; p.W_min = 1; p.W_cap = W_S; p.t = -1.0f; p.top_k = top_k; p.top_p = top_p;
  return p;
}

int32_t check_draft(const dsbd_draft_in* in, int32_t W_S) {
  if (!in) return DSBD_ERR_INVALID;
  if (in->n_prompts < 0 || in->n_beams < 0 || in->max_prompt_beams < 0) return DSBD_ERR_INVALID;
  if (W_S < 1 || W_S > 64 || in->max_prompt_beams > 64) return DSBD_ERR_UNSUPPORTED;
  if (in->V < 1) return DSBD_ERR_UNSUPPORTED;
  return DSBD_OK;
}

size_t carve_draft(WorkspaceCarver& ws, const dsbd_draft_in* in, int32_t W_S, size_t verify_bytes, DraftScratch* s) {
  const size_t B = (size_t)in->n_beams, P = (size_t)in->n_prompts;
  s->tree_prompt = ws.take<int32_t>(B);
  s->tree_off = ws.take<int32_t>(B + 1);
  s->parent = ws.take<int32_t>(B);
  s->token = ws.take<int32_t>(B);
  s->u_accept = ws.take<float>(B);
  s->u_resid = ws.take<float>(2 * P);
  s->u_fill = ws.take<float>(2 * P * W_S);
  s->node_status = ws.take<uint8_t>(B);
  s->l_last = ws.take<int32_t>(P);
  s->layer_width = ws.take<int32_t>(2 * P);
  s->n_out = ws.take<int32_t>(P);
  s->out_node = ws.take<int32_t>(P * W_S);
  s->near_tie = ws.take<int32_t>(P);
  s->out_logp_other = ws.take<double>(P * W_S);
  s->verify_ws = ws.take<char>(verify_bytes);
  return ws.total();
}

}  // namespace

extern "C" size_t dsbd_draft_layer_workspace_bytes(const dsbd_draft_in* in, int32_t W_S, int32_t top_k, float top_p) {
  if (check_draft(in, W_S) != DSBD_OK) return 0;
  if (in->n_beams == 0 || in->n_prompts == 0) return 256;
  DraftScratch s;
  dsbd_forest f;
  WorkspaceCarver none(nullptr);
  carve_draft(none, in, W_S, 0, &s);
  make_forest(in, s, &f);
  const dsbd_params p = make_params(W_S, top_k, top_p);
  const size_t vb = dsbd_verify_forest_workspace_bytes(&f, in->V, &p);
  if (vb == 0) return 0;
  WorkspaceCarver ws(nullptr);
  return carve_draft(ws, in, W_S, vb, &s) + 256;
}

extern "C" int32_t dsbd_draft_layer(const dsbd_draft_in* in, int32_t W_S, int32_t top_k, float top_p,
                                    const dsbd_draft_out* out, void* workspace, size_t workspace_bytes,
                                    int32_t* fault, void* stream_) {
  if (!out || !fault) return DSBD_ERR_INVALID;
  const int32_t rc = check_draft(in, W_S);
  if (rc != DSBD_OK) return rc;
  if (in->n_beams == 0 || in->n_prompts == 0) return DSBD_OK;
  if (!in->beam_off || !in->logits_draft || !in->beam_logp_draft || !in->u) return DSBD_ERR_INVALID;
  if (!out->parent || !out->token || !out->logp_draft || !workspace) return DSBD_ERR_INVALID;
  const size_t need = dsbd_draft_layer_workspace_bytes(in, W_S, top_k, top_p);
  if (need == 0) return DSBD_ERR_UNSUPPORTED;
  if (workspace_bytes < need) return DSBD_ERR_WORKSPACE;
  hipStream_t stream = static_cast<hipStream_t>(stream_);

  DraftScratch s;
  dsbd_forest f;
  const dsbd_params p = make_params(W_S, top_k, top_p);
  {
    WorkspaceCarver none(nullptr);
    carve_draft(none, in, W_S, 0, &s);
    make_forest(in, s, &f);
  }
  const size_t vb = dsbd_verify_forest_workspace_bytes(&f, in->V, &p);
  char* wbase = reinterpret_cast<char*>(dsbd_align_up(reinterpret_cast<uintptr_t>(workspace), 256));
  WorkspaceCarver ws(wbase);
  carve_draft(ws, in, W_S, vb, &s);
  make_forest(in, s, &f);

  DraftSetupArgs sa;
  sa.n_prompts = in->n_prompts; sa.n_beams = in->n_beams; sa.W_S = W_S;
  sa.beam_off = in->beam_off; sa.u = in->u;
  sa.tree_prompt = s.tree_prompt; sa.tree_off = s.tree_off; sa.parent = s.parent; sa.token = s.token;
  sa.u_accept = s.u_accept; sa.u_resid = s.u_resid; sa.u_fill = s.u_fill; sa.fault = fault;
  long long items = in->n_beams + 1;
  if (items < 2LL * in->n_prompts * W_S) items = 2LL * in->n_prompts * W_S;
  hipLaunchKernelGGL(draft_setup_kernel, dim3((unsigned)((items + DR_BLOCK - 1) / DR_BLOCK)), dim3(DR_BLOCK), 0, stream, sa);
  DSBD_HIP_LAUNCH_CHECK();

  dsbd_verify_in vin;
  vin.V = in->V;
  vin.logits_target = in->logits_draft; vin.logits_draft = in->logits_draft;      // one model in both roles
  vin.beam_logp_target = in->beam_logp_draft; vin.beam_logp_draft = in->beam_logp_draft;
  vin.u_accept = s.u_accept; vin.u_resid = s.u_resid; vin.u_fill = s.u_fill;
  dsbd_verify_out vout = {};
  vout.node_status = s.node_status; vout.l_last = s.l_last; vout.layer_width = s.layer_width; vout.n_out = s.n_out;
  vout.out_parent = out->parent; vout.out_token = out->token; vout.out_node = s.out_node;
  vout.out_logp_target = out->logp_draft; vout.out_logp_draft = s.out_logp_other;
  vout.near_tie_count = s.near_tie;
  return dsbd_verify_forest(&f, &vin, &p, &vout, s.verify_ws, vb, fault, stream_);
}

// ------------------------------------------------------------------------------------------------ forest layout
namespace {

struct BuildArgs {
  int n_prompts, n_roots, gamma, W_S;
  const int32_t *root_off, *root_token, *layer_parent, *layer_token;
  dsbd_forest_out out;
  int32_t* fault;
};

struct BuildShared {
  int root[BF_NODE_CAP];        // prompt-local input beam every node descends from
  int key[BF_NODE_CAP];         // layer * W_S + draw index (0 for roots): the order inside a tree
  int par_local[BF_NODE_CAP];   // prompt-local index (layer-major) of the parent, -1 for roots
  int pos[BF_NODE_CAP];         // position of the node in the prompt's part of the forest
  int tree_n[64];
  int bad;
};

__global__ __launch_bounds__(BF_BLOCK) void build_forest_kernel(BuildArgs a) {
  __shared__ BuildShared sh;
  const int p = blockIdx.x, tid = threadIdx.x;
  const int r0 = a.root_off[p], r1 = a.root_off[p + 1];
  int W = r1 - r0;
  const int rows = a.n_prompts * a.W_S;                 // rows of a drafted layer
  int bad = 0;
  if (r0 < 0 || r1 > a.n_roots || W < 0 || W > 64) { bad |= DSBD_FAULT_BOUNDS; W = 0; }
  if (p == 0 && r0 != 0) bad |= DSBD_FAULT_TOPOLOGY;
  if (p == a.n_prompts - 1 && r1 != a.n_roots) bad |= DSBD_FAULT_TOPOLOGY;
  int n_p = W > 0 ? W + a.gamma * a.W_S : 0;            // nodes of the prompt; local index: roots, then layer-major
  if (n_p > BF_NODE_CAP) { bad |= DSBD_FAULT_BOUNDS; n_p = 0; W = 0; }
  const long long base = (long long)r0 + (long long)p * a.gamma * a.W_S;     // first forest node of the prompt
  if (tid == 0) sh.bad = 0;
  if (tid < 64) sh.tree_n[tid] = 0;
  __syncthreads();
  // every node: its parent (prompt-local) and, walking up, its input beam
  if (tid < n_p) {
    int l = 0, j = tid, par = -1, root = tid;
    if (tid >= W) {
      l = 1 + (tid - W) / a.W_S; j = (tid - W) % a.W_S;
      int cur_l = l, row = p * a.W_S + j;
      while (cur_l >= 1) {
        int up = a.layer_parent[(long long)(cur_l - 1) * rows + row];
        // rows of the layer above that belong to this prompt
        const int lo = cur_l == 1 ? r0 : p * a.W_S, hi = cur_l == 1 ? r1 : (p + 1) * a.W_S;
        if (up < lo || up >= hi) { atomicOr(&sh.bad, DSBD_FAULT_TOPOLOGY); up = lo; }
        if (cur_l == l) par = cur_l == 1 ? up - r0 : W + (cur_l - 2) * a.W_S + (up - p * a.W_S);
        row = up;
        cur_l -= 1;
      }
      root = row - r0;
    }
    sh.root[tid] = root;
    sh.key[tid] = tid < W ? 0 : l * a.W_S + j;          // a root comes first in its tree (its own index may exceed W_S)
    sh.par_local[tid] = par;
    atomicAdd(&sh.tree_n[root], 1);
  }
  __syncthreads();
  if (tid < n_p) {
    const int root = sh.root[tid], key = sh.key[tid];
    int pos = 0;
    for (int c = 0; c < n_p; ++c) {
      const int rc = sh.root[c], kc = sh.key[c];
      pos += (rc < root) | ((rc == root) & (kc < key));
    }
    sh.pos[tid] = pos;
  }
  __syncthreads();
  if (tid < n_p) {
    const long long n = base + sh.pos[tid];
    const int par = sh.par_local[tid];
    a.out.parent[n] = par < 0 ? -1 : (int)(base + sh.pos[par]);
    if (tid < W) {
      a.out.token[n] = a.root_token ? a.root_token[r0 + tid] : 0;
      a.out.draft_rank[n] = 0;
      a.out.tree_prompt[r0 + tid] = p;
      a.out.tree_off[r0 + tid] = (int)n;
      a.out.node_of_root[r0 + tid] = (int)n;
      if (sh.tree_n[tid] > DSBD_MAX_TREE_NODES) atomicOr(&sh.bad, DSBD_FAULT_BOUNDS);
      atomicMax(a.out.max_tree_nodes, sh.tree_n[tid]);
    } else {
      const int l = 1 + (tid - W) / a.W_S, j = (tid - W) % a.W_S;
      const long long li = (long long)(l - 1) * rows + p * a.W_S + j;
      a.out.token[n] = a.layer_token[li];
      a.out.draft_rank[n] = j;
      a.out.node_of[li] = (int)n;
    }
  }
  if (W == 0 && n_p == 0) {
    // a prompt without input beams (or one that does not fit): its draws get no node
    for (int i = tid; i < a.gamma * a.W_S; i += BF_BLOCK) {
      const int l = 1 + i / a.W_S, j = i % a.W_S;
      a.out.node_of[(long long)(l - 1) * rows + p * a.W_S + j] = -1;
    }
  }
  if (p == a.n_prompts - 1 && tid == 0) a.out.tree_off[a.n_roots] = a.n_roots + a.gamma * rows;
  __syncthreads();
  if (tid == 0 && (bad | sh.bad)) atomicOr(a.fault, bad | sh.bad);
}

__global__ void build_forest_init_kernel(int32_t* max_tree_nodes) { *max_tree_nodes = 0; }

}  // namespace

extern "C" int32_t dsbd_build_forest(int32_t n_prompts, int32_t n_roots, int32_t gamma, int32_t W_S,
                                     const int32_t* root_off, const int32_t* root_token,
                                     const int32_t* layer_parent, const int32_t* layer_token,
                                     const dsbd_forest_out* out, int32_t* fault, void* stream_) {
  if (!out || !fault) return DSBD_ERR_INVALID;
  if (n_prompts < 0 || n_roots < 0 || gamma < 0 || W_S < 0) return DSBD_ERR_INVALID;
  if (gamma > 0 && (W_S < 1 || W_S > 64)) return DSBD_ERR_UNSUPPORTED;
  if (gamma >= DSBD_MAX_TREE_NODES) return DSBD_ERR_UNSUPPORTED;
  if (n_prompts == 0) return DSBD_OK;
  if (!root_off || (gamma > 0 && (!layer_parent || !layer_token))) return DSBD_ERR_INVALID;
  if (!out->tree_prompt || !out->tree_off || !out->parent || !out->token || !out->draft_rank || !out->node_of_root ||
      !out->max_tree_nodes || (gamma > 0 && !out->node_of))
    return DSBD_ERR_INVALID;
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  BuildArgs a;
  a.n_prompts = n_prompts; a.n_roots = n_roots; a.gamma = gamma; a.W_S = gamma > 0 ? W_S : 0;
  a.root_off = root_off; a.root_token = root_token; a.layer_parent = layer_parent; a.layer_token = layer_token;
  a.out = *out; a.fault = fault;
  hipLaunchKernelGGL(build_forest_init_kernel, dim3(1), dim3(1), 0, stream, out->max_tree_nodes);
  hipLaunchKernelGGL(build_forest_kernel, dim3((unsigned)n_prompts), dim3(BF_BLOCK), 0, stream, a);
  DSBD_HIP_LAUNCH_CHECK();
  return DSBD_OK;
}
