// Physical key/value cache update after an iteration (paper Section 3.3, last paragraph: the caches are
// updated to follow the output beams; Section 3.4: a single cache in the memory-reduced variant).
//
// The cache of a next-iteration beam = the own cache segment of the input beam it descends from, followed by the
// key/value rows of the forest nodes on the path root .. the node the output beam hangs from (the plan written by
// dsbd_select_beams).  A pure copy, bound by HBM bandwidth: one workgroup per (destination beam, K or V, chunk of
// 16 tokens), 16-byte pieces, four loads in flight per thread.  A destination that IS its source buffer (the beam
// continues in place) only gets the tree rows appended.
#include "common.h"

#define CM_BLOCK 256
#define CM_TOKENS 16           // tokens per workgroup (measured: 16 -> 72 us, 64 -> 79 us, 128 -> 115 us on the benchmark plan)

struct CommitArgs {
  int n_prompts, n_trees, n_nodes, W_cap, plen, Hkv, D;
  const void* const* src_k; const void* const* src_v; const int32_t* src_len;
  long long token_stride, head_stride;      // elements; the same layout for sources and destinations
  const __bf16 *k_tree, *v_tree;            // [n_nodes, Hkv, D]
  const int32_t *n_next, *src_tree, *path_len, *path;
  void* const* dst_k; void* const* dst_v; int32_t* dst_len;
  int capacity, max_len;
  int32_t* fault;
};

typedef unsigned int cm_u32x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(1))) cm_u32x4 cm_gvec;

__global__ __launch_bounds__(CM_BLOCK) void commit_kv_kernel(CommitArgs a) {
  const int chunk = blockIdx.x, j = blockIdx.y, is_v = blockIdx.z;
  const int tid = threadIdx.x;
  const int p = j / a.W_cap, s = j % a.W_cap;
  const bool speaker = chunk == 0 && is_v == 0 && tid == 0;     // one thread per destination reports and writes the length
  int nn = a.n_next[p];
  nn = max(0, min(nn, a.W_cap));
  if (s >= nn) { if (speaker) a.dst_len[j] = 0; return; }
  const int b = a.src_tree[j];
  if (b < 0 || b >= a.n_trees) {
    if (speaker) { a.dst_len[j] = 0; atomicOr(a.fault, DSBD_FAULT_TOPOLOGY); }
    return;
  }
  // the source length is the caller's: the grid covers max_len + path tokens, so a longer source cannot be copied
  const int L_raw = a.src_len[b];
  const int L = max(0, min(L_raw, a.max_len));
  const int pl = max(0, min(a.path_len[j], a.plen));
  const int total = L + pl;
  // Both planes are checked by every workgroup (the K and the V workgroups of a destination must take the same
  // decision: a destination with a usable K buffer and a null or misaligned V buffer is left untouched as a whole).
  const char* src_kp = static_cast<const char*>(a.src_k[b]);
  const char* src_vp = static_cast<const char*>(a.src_v[b]);
  char* dst_kp = static_cast<char*>(a.dst_k[j]);
  char* dst_vp = static_cast<char*>(a.dst_v[j]);
  const bool bad = L_raw < 0 || L_raw > a.max_len || total > a.capacity || !dst_kp || !dst_vp ||
                   (L > 0 && (!src_kp || !src_vp)) ||
                   ((reinterpret_cast<uintptr_t>(dst_kp) | reinterpret_cast<uintptr_t>(src_kp) |
                     reinterpret_cast<uintptr_t>(dst_vp) | reinterpret_cast<uintptr_t>(src_vp)) & 15);
  const char* src = is_v ? src_vp : src_kp;
  char* dst = is_v ? dst_vp : dst_kp;
  if (bad) {      // uniform over the destination's workgroups: the destination is left untouched
    if (speaker) { a.dst_len[j] = 0; atomicOr(a.fault, DSBD_FAULT_BOUNDS); }
    return;
  }
  if (speaker) a.dst_len[j] = total;
  const int t0 = chunk * CM_TOKENS;
  const int t1 = min(total, t0 + CM_TOKENS);
  if (t0 >= t1) return;
  const bool in_place = dst == src;          // the beam keeps its buffer: only the tree rows are appended
  const __bf16* rows = is_v ? a.v_tree : a.k_tree;
  const int CG = a.D / 8;                    // 16-byte pieces per (token, head)
  const int per_tok = a.Hkv * CG;
  const int n_piece = (t1 - t0) * per_tok;
  auto src_of = [&](int piece, long long& doff) -> const char* {
    const int t = t0 + piece / per_tok;
    const int r = piece % per_tok;
    const int g = r / CG, c = r % CG;
    doff = ((long long)t * a.token_stride + (long long)g * a.head_stride + c * 8) * 2;
    if (t < L) return in_place ? nullptr : src + doff;
    int node = a.path[(long long)j * a.plen + (t - L)];
    if (node < 0 || node >= a.n_nodes) { atomicOr(a.fault, DSBD_FAULT_TOPOLOGY); return nullptr; }
    return reinterpret_cast<const char*>(rows + ((long long)node * a.Hkv + g) * a.D + c * 8);
  };
  for (int i0 = tid; i0 < n_piece; i0 += 4 * CM_BLOCK) {
    cm_u32x4 v[4];
    long long doff[4];
    bool have[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const int i = i0 + k * CM_BLOCK;
      have[k] = false;
      if (i < n_piece) {
        const char* sp = src_of(i, doff[k]);
        // plain loads (several next beams usually copy the same source: let the caches serve the repeats),
        // non-temporal stores (the copies are not read again before the next iteration)
        if (sp) { v[k] = *(const cm_gvec*)(sp); have[k] = true; }
      }
    }
#pragma unroll
    for (int k = 0; k < 4; ++k)
      if (have[k]) __builtin_nontemporal_store(v[k], (cm_gvec*)(dst + doff[k]));
  }
}

extern "C" int32_t dsbd_commit_kv(const dsbd_forest* f, const dsbd_kv* src, const void* k_tree, const void* v_tree,
                                  int32_t Hkv, int32_t D, const dsbd_next_beams* next, int32_t W_cap,
                                  const dsbd_kv_dst* dst, int32_t* fault, void* stream_) {
  if (!f || !src || !next || !dst || !fault) return DSBD_ERR_INVALID;
  if (W_cap < 1 || W_cap > 64) return DSBD_ERR_UNSUPPORTED;
  if (Hkv <= 0 || D <= 0 || D % 8 != 0) return DSBD_ERR_UNSUPPORTED;
  if (f->max_depth < 0 || f->max_depth >= DSBD_MAX_TREE_NODES) return DSBD_ERR_INVALID;
  if (f->n_prompts < 0 || f->n_trees < 0 || f->n_nodes < 0 || src->max_len < 0 || dst->capacity < 0) return DSBD_ERR_INVALID;
  if (src->token_stride % 8 != 0 || src->head_stride % 8 != 0) return DSBD_ERR_UNSUPPORTED;
  if (f->n_prompts == 0) return DSBD_OK;
  if (!src->k_ptr || !src->v_ptr || !src->len || !k_tree || !v_tree) return DSBD_ERR_INVALID;
  if (!next->n_next || !next->src_tree || !next->path_len || !next->path) return DSBD_ERR_INVALID;
  if (!dst->k_ptr || !dst->v_ptr || !dst->len) return DSBD_ERR_INVALID;
  if ((reinterpret_cast<uintptr_t>(k_tree) | reinterpret_cast<uintptr_t>(v_tree)) & 15) return DSBD_ERR_INVALID;
  CommitArgs a;
  a.n_prompts = f->n_prompts; a.n_trees = f->n_trees; a.n_nodes = f->n_nodes; a.W_cap = W_cap;
  a.plen = f->max_depth + 1; a.Hkv = Hkv; a.D = D;
  a.src_k = src->k_ptr; a.src_v = src->v_ptr; a.src_len = src->len;
  a.token_stride = src->token_stride; a.head_stride = src->head_stride;
  a.k_tree = static_cast<const __bf16*>(k_tree); a.v_tree = static_cast<const __bf16*>(v_tree);
  a.n_next = next->n_next; a.src_tree = next->src_tree; a.path_len = next->path_len; a.path = next->path;
  a.dst_k = dst->k_ptr; a.dst_v = dst->v_ptr; a.dst_len = dst->len; a.capacity = dst->capacity; a.max_len = src->max_len;
  a.fault = fault;
  const long long max_tokens = (long long)src->max_len + a.plen;
  const long long chunks = (max_tokens + CM_TOKENS - 1) / CM_TOKENS;
  const long long slots = (long long)f->n_prompts * W_cap;
  if (chunks > 0x7fffffffLL || slots > 65535) return DSBD_ERR_UNSUPPORTED;
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  dsbd_launch(DSBD_KERNEL_KV_COMMIT, commit_kv_kernel, dim3((unsigned)chunks, (unsigned)slots, 2), dim3(CM_BLOCK), 0, stream, a);
  DSBD_HIP_LAUNCH_CHECK();
  return DSBD_OK;
}
