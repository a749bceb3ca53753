// Layer-wise verification of a draft forest on gfx950 (paper Section 3.1 "Details", Algorithm 1,
// and the dynamic layer width of Section 3.2, Eq. 1-6).
//
// Two kernels that do not depend on each other and run side by side (the layer kernel on the caller's stream, the
// statistics pass on a second stream of the library's own, forked from and joined to the caller's):
//
// 1. vocab_stats_kernel + vocab_finish_kernel (bandwidth-bound, all nodes, both models): one pass over the fp32 logits
//    with a per-thread online max / sum-of-exponentials, reduced per row chunk, then per node the fp32 log-sum-exp and
//    the log-probability of the node's own token under its parent.  This is the O(W |V|) softmax work of the
//    beam-sampling joint (Section 2.1) done once for every forest node; it feeds the per-node outputs only.
// 2. verify_layers_kernel (latency-bound, persistent; all its workgroups must be resident at once): G workgroups per
//    prompt walk the layers in order.  Every decision is taken in fp64.  The kernel derives everything from the call's
//    inputs (tree and node range of its prompt, node depths, the maxima and sums of the rows it uses).  For the
//    layer's input beams I the workgroups materialise p_beam and q_beam over I x V (their slice each), and every
//    dependent reduction over I x V is one pass over the slices plus one exchange among the G workgroups.
//
// The running residual p' is never stored.  After k consecutive rejections since the last reset
//     p'_k = max(p_beam - c_k q_beam, 0) / F(c_k),   F(c) = sum max(p_beam - c q_beam, 0),
//     c_1 = 0, F(c_1) := 1, c_{k+1} = c_k + F(c_k)
// (induction on p'_{k+1} = norm(max(0, p'_k - q_beam))), so a rejection costs one evaluation of F, the
// chain {c_k, F(c_k)} depends only on (p_beam, q_beam) and is reused after every acceptance resets p'
// to p_beam, and the conditional acceptance probabilities of Eq. 3 are alpha_k = 1 - F(c_{k+1})/F(c_k).
//
// All G workgroups of a prompt run the same sequential program on the same reduced values (summed in
// the same order), so their control flow stays identical without any broadcast.
#include "common.h"
#include "topology_device.h"
#include "exp_nonpos.h"
#include <type_traits>
#include <float.h>
#include <limits.h>
#include <stdlib.h>
#include <atomic>
#include <mutex>

#define VS_BLOCK 256
#define VL_BLOCK 512
#define NODE_CAP 512           // nodes of one prompt (all its trees)
#define NEAR_TIE 1.0e-6
#define SYNC_LIMIT_TICKS 300000000LL   // default bound of every wait: 3 s of the 100 MHz wall clock
#define DSBD_STATIC_SCRATCH_BYTES (32u << 20)   // the device array behind dsbd_verify_forest_static
#define CU_LDS_BYTES (160 * 1024)  // LDS of a compute unit (gfx950)
#define STATS_SIDE_WGS 1        // workgroups of the statistics pass per compute unit beside the layer kernel
#define XU 4                   // logits per thread and model in flight in the exponential pass.  Eight (a 4008-entry piece of the
                               // benchmark's joint in one round) cost 256 vector registers; with four the kernel needs 186,
                               // which leaves room on every SIMD for waves of the statistics pass running beside it
#define VL_DYN_LDS_BYTES (80 * 1024)   // dynamic LDS of the layer kernel (its static LDS takes most of the rest) ...
#define VL_DYN_LDS_BYTES_SMALL (112 * 1024)   // ... and of its variant for prompts of at most NODE_CAP_SMALL nodes
#define NODE_CAP_SMALL 128

// ------------------------------------------------------------------------------------------------ kernel 1
struct StatsArgs {
  const float* z[2];
  int n_nodes, V, nchunk, chunk;
  float2* part;      // [2][n_nodes][nchunk] (max, sum of exp(x - max))
  int32_t* fault;
};

// 2^x by the hardware instruction alone: results below 2^-126 come out as zero instead of denormal, which a sum
// of terms relative to the running maximum does not notice (the library routine spends four more instructions
// per logit on that range).
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ __forceinline__ void online_add4(float& m, float& s, bool& bad, float x0, float x1, float x2, float x3) {
  const float L2E = 1.4426950408889634f;
  const float bm = fmaxf(fmaxf(x0, x1), fmaxf(x2, x3));
  bad |= !(x0 <= FLT_MAX) | !(x1 <= FLT_MAX) | !(x2 <= FLT_MAX) | !(x3 <= FLT_MAX);      // NaN or +Inf (-Inf: a masked token)
  if (bm > m) {
    s *= fast_exp2((m - bm) * L2E);
    m = bm;
  }
  const float ref = m == -INFINITY ? 0.f : m;       // (nothing but masked tokens so far: they add 0, not exp(-Inf + Inf))
  s += fast_exp2((x0 - ref) * L2E) + fast_exp2((x1 - ref) * L2E) + fast_exp2((x2 - ref) * L2E) + fast_exp2((x3 - ref) * L2E);
}

__device__ __forceinline__ void online_add16(float& m, float& s, bool& bad, float4 a, float4 b, float4 c, float4 d) {
  const float L2E = 1.4426950408889634f;
  const float v[16] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w, c.x, c.y, c.z, c.w, d.x, d.y, d.z, d.w};
  float bm = v[0];
#pragma unroll
  for (int e = 1; e < 16; ++e) bm = fmaxf(bm, v[e]);
  bool nan = false;
#pragma unroll
  for (int e = 0; e < 16; ++e) nan |= (v[e] != v[e]);
  bad |= nan | !(bm <= FLT_MAX);                     // NaN or +Inf (-Inf: a masked token, probability 0)
  if (bm > m) {
    s *= fast_exp2((m - bm) * L2E);
    m = bm;
  }
  const float ref = m == -INFINITY ? 0.f : m;       // (nothing but masked tokens so far: they add 0, not exp(-Inf + Inf))
  float t0 = 0.f, t1 = 0.f, t2 = 0.f, t3 = 0.f;
#pragma unroll
  for (int e = 0; e < 16; e += 4) {
    t0 += fast_exp2((v[e] - ref) * L2E); t1 += fast_exp2((v[e + 1] - ref) * L2E);
    t2 += fast_exp2((v[e + 2] - ref) * L2E); t3 += fast_exp2((v[e + 3] - ref) * L2E);
  }
  s += (t0 + t1) + (t2 + t3);
}

__device__ __forceinline__ void online_add1(float& m, float& s, bool& bad, float x) {
  const float L2E = 1.4426950408889634f;
  bad |= !(x <= FLT_MAX);                            // NaN or +Inf
  if (x > m) {
    s *= fast_exp2((m - x) * L2E);
    m = x;
  }
  s += fast_exp2((x - (m == -INFINITY ? 0.f : m)) * L2E);
}

__device__ __forceinline__ void online_merge(float& m, float& s, float m2, float s2) {
  const float L2E = 1.4426950408889634f;
  const float mn = fmaxf(m, m2);
  if (mn == -INFINITY) { s = 0.f; return; }
  s = s * exp2f((m - mn) * L2E) + s2 * exp2f((m2 - mn) * L2E);
  m = mn;
}

__global__ __launch_bounds__(VS_BLOCK) void vocab_stats_kernel(StatsArgs a) {
  const int c = blockIdx.x, n = (int)blockIdx.y, which = blockIdx.z;
  const int lo = c * a.chunk;
  const int hi = min(a.V, lo + a.chunk);
  const float* row = a.z[which] + (long long)n * a.V;
  float m = -INFINITY, s = 0.f;
  bool bad = false;
  // scalar head up to 16-byte alignment, float4 body, scalar tail
  const uintptr_t addr = reinterpret_cast<uintptr_t>(row + lo);
  int head = (int)(((16 - (addr & 15)) & 15) >> 2);
  head = min(head, hi - lo);
  const int body4 = (hi - lo - head) >> 2;
  const int tail0 = lo + head + 4 * body4;
  if ((int)threadIdx.x < head) online_add1(m, s, bad, row[lo + threadIdx.x]);
  const float4* r4 = reinterpret_cast<const float4*>(row + lo + head);
  typedef float f32x4 __attribute__((ext_vector_type(4)));
  const f32x4* n4 = reinterpret_cast<const f32x4*>(r4);
  int i = threadIdx.x;
  // four 16-byte loads in flight per thread (the pass is bound by memory latency x bytes in flight), and one
  // rescaling of the running sum per sixteen logits instead of one per four
  for (; i + 3 * VS_BLOCK < body4; i += 4 * VS_BLOCK) {
    // streamed once: non-temporal loads keep the 250 MB pass from churning the caches (measured 15 % faster)
    const f32x4 y0 = __builtin_nontemporal_load(&n4[i]), y1 = __builtin_nontemporal_load(&n4[i + VS_BLOCK]),
                y2 = __builtin_nontemporal_load(&n4[i + 2 * VS_BLOCK]), y3 = __builtin_nontemporal_load(&n4[i + 3 * VS_BLOCK]);
    const float4 x0 = make_float4(y0.x, y0.y, y0.z, y0.w), x1 = make_float4(y1.x, y1.y, y1.z, y1.w),
                 x2 = make_float4(y2.x, y2.y, y2.z, y2.w), x3 = make_float4(y3.x, y3.y, y3.z, y3.w);
    online_add16(m, s, bad, x0, x1, x2, x3);
  }
  if (i < body4) {
    // the ragged last group, its loads in flight together as well (one after the other they cost a memory latency
    // each at the end of every workgroup); the places beyond the end hold the most negative finite number, which
    // changes neither the maximum nor the sum and is no fault
    f32x4 y[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) y[k] = __builtin_nontemporal_load(&n4[min(i + k * VS_BLOCK, body4 - 1)]);
    float4 x[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const bool in = i + k * VS_BLOCK < body4;
      x[k] = in ? make_float4(y[k].x, y[k].y, y[k].z, y[k].w) : make_float4(-FLT_MAX, -FLT_MAX, -FLT_MAX, -FLT_MAX);
    }
    online_add16(m, s, bad, x[0], x[1], x[2], x[3]);
  }
  if (tail0 + (int)threadIdx.x < hi) online_add1(m, s, bad, row[tail0 + threadIdx.x]);

  // block reduction
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    const float m2 = __shfl_xor(m, off), s2 = __shfl_xor(s, off);
    online_merge(m, s, m2, s2);
  }
  __shared__ float sm[VS_BLOCK / 64], ss[VS_BLOCK / 64];
  __shared__ int sbad;
  if (threadIdx.x == 0) sbad = 0;
  __syncthreads();
  if (bad) sbad = 1;
  if ((threadIdx.x & 63) == 0) { sm[threadIdx.x >> 6] = m; ss[threadIdx.x >> 6] = s; }
  __syncthreads();
  if (threadIdx.x == 0) {
    float M = sm[0], S = ss[0];
    for (int w = 1; w < VS_BLOCK / 64; ++w) online_merge(M, S, sm[w], ss[w]);
    a.part[((long long)which * a.n_nodes + n) * a.nchunk + c] = make_float2(M, S);
    if (sbad) atomicOr(a.fault, DSBD_FAULT_NONFINITE);
  }
}

// Per-node outputs of the statistics pass: the chunks of a row merged into its fp32 log-sum-exp, and the
// log-probability of each node's own token under its parent's row (Section 2.1: the likelihood a beam stores grows by
// this term).  One thread per node; the parent's chunks are merged again by the child (a handful of values).
struct FinishArgs {
  const float* z[2];
  int n_nodes, V, nchunk, alias;
  const float2* part;
  const int32_t *parent, *token;
  float *lse[2], *logp[2];     // outputs (any may be null)
  int32_t* fault;
};

__device__ __forceinline__ float merged_lse(const float2* pp, int nchunk) {
  float M = pp[0].x, S = pp[0].y;
  for (int c = 1; c < nchunk; ++c) online_merge(M, S, pp[c].x, pp[c].y);
  return M + logf(S);
}

__global__ __launch_bounds__(VS_BLOCK) void vocab_finish_kernel(FinishArgs a) {
  const int n = blockIdx.x * VS_BLOCK + threadIdx.x;
  if (n >= a.n_nodes) return;
  const int par = a.parent[n];
  const int tok = a.token[n];
  const bool has_parent = par >= 0 && par < n && tok >= 0 && tok < a.V;
#pragma unroll
  for (int m = 0; m < 2; ++m) {
    const float2* base = a.part + (a.alias ? 0 : (long long)m * a.n_nodes * a.nchunk);
    const float own = merged_lse(base + (long long)n * a.nchunk, a.nchunk);
    if (own == -INFINITY) atomicOr(a.fault, DSBD_FAULT_NONFINITE);     // a row without a finite logit
    if (a.lse[m]) a.lse[m][n] = own;
    // A masked logit (-Inf) is a token of probability 0, but not at a drafted token: its beam would carry the
    // likelihood 0, and a layer whose beams all do has no joint.  Reported like the other non-finite logits.
    const float zt = has_parent ? a.z[m][(long long)par * a.V + tok] : 0.f;
    if (zt == -INFINITY) atomicOr(a.fault, DSBD_FAULT_NONFINITE);
    if (a.logp[m]) {
      float lp = 0.f;
      if (has_parent) lp = zt - merged_lse(base + (long long)par * a.nchunk, a.nchunk);
      a.logp[m][n] = lp;
    }
  }
}

// ------------------------------------------------------------------------------------------------ kernel 2
// Where the exchanges of one prompt keep their 16-byte slots (offsets in slots from the prompt's first one).
struct SlotLayout {
  int x[2];              // the two alternating banks of the post-then-collect-from-all exchanges: G lines
  int xc[2];             // ... and of the group sums of their two-hop form: SUM_GROUPS lines
  int r, r_w, r_stride;  // row sums of layer l: r + (l - 1) * r_stride, r_w slots per workgroup
  int s, s_stride;       // early chain entry of layer l: s + (l - 1) * s_stride, a line per workgroup
  int sc, sc_stride;     // its group sums: sc + (l - 1) * sc_stride, SUM_GROUPS lines
  int b, b_w;            // warping: every workgroup's candidate list, b_w slots each
  int c;                 // warping: the groups' merged lists (b_w slots each)
  int d;                 // warping: the final entries, posted by the prompt's first workgroup
  int wb, wb_stride;     // warping, one-level form: the workgroups' candidates of layer l at wb + (l - 1) * wb_stride, b_w
                         // slots per workgroup (two counts, then value | index)
  int acc;               // accumulator words of the one-hop sums: 2 banks x NACC lines
  int acc0;              // their values at launch, posted by the prompt's first workgroup: 2 x NACC slots
  int prompt_stride;
};
#define WARP_RESULT_SLOTS 193     // count + 64 x (index, p, q)

struct LayersArgs {
  int n_prompts, n_trees, n_nodes;
  const int32_t *tree_prompt, *tree_off, *parent, *token, *rank;
  int max_depth, max_prompt_trees;
  int V;
  const float *zp, *zq;
  const double *blp, *blq;
  const float *u_acc, *u_res, *u_fill;
  int W_L, W_min, W_cap;
  float t;
  int top_k;             // warping T (Section 2.1): keep the top_k largest entries of each joint (0: T is the identity) ...
  float top_p;           // ... then the smallest leading part of those whose share of the kept mass exceeds top_p
  dsbd_verify_out out;
  int prompt0;           // first prompt of this launch (forests of more prompts than fit the device run in groups)
  int max_tree_nodes;
  double* pb;            // [n_prompts][G][slice_cap]  p_beam slice storage, a private region per workgroup
  double* qb;            // the same for q_beam
  long long slice_cap;   // elements of a workgroup's region
  double* red;           // exchange slots of 16 bytes each, n_prompts regions laid out as in `sl`
  SlotLayout sl;
  int G, I_cap;
  long long* trace;      // optional timeline of workgroup trace_wg: pairs (label, 100 MHz wall clock)
  int trace_wg;
  int lds_elems;         // capacity (elements) of each of the two dynamic-LDS slice arrays; 0 = none
  int lds_slice;         // slices of up to this many elements are kept in the LDS (<= lds_elems)
  int alias;             // one model in both roles (same logits, same beam likelihoods): q_beam IS p_beam, kept once
  long long sync_limit;  // bound of every wait, in ticks of the 100 MHz wall clock
  unsigned long long nonce;   // base of this launch's exchange tags: no tag of an earlier launch on the same workspace can match
  const unsigned long long* replay;   // launches recorded into a graph: a word of the workspace that a small kernel in front of
                              // this one counts up at every replay (the arguments, nonce included, repeat); else null
  int mute_wg;           // test hook: this workgroup withholds its first post (-1: none), so that its partners'
                         // bounded waits give up and the error path can be exercised without a hang
  int32_t* fault;
  int warp_fast;         // warping: the one-level selection (bounds from the workgroups' largest entries) where it applies
  dsbd_next_beams nx;    // next-beam plan written along with the output beams (fused selection) ...
  int nx_on;             // ... when this is set
};

#define VL_WAVES (VL_BLOCK / 64)
#define NODE_DEPTH_MASK 0xff   // LayerShared::n_depth: depth of the node (below 64) ...
#define NODE_TREE_SHIFT 8      // ... and, above it, the index of its tree among the prompt's trees (below 64)
#define NACC 8                 // accumulator words of a one-hop sum (see wave_sum_accumulators)
#define ACC_FIELD_BITS 54
static_assert(NODE_CAP <= VL_BLOCK, "one thread per node of a prompt");
static_assert(VL_WAVES == 8, "the fixed reduction trees below are written for eight waves");

// NC: the most nodes a prompt may have (all its trees).  Two sizes are built: what the arrays below do not take of a
// compute unit's LDS is room for the joint slices.
template <int NC>
struct LayerShared {
  // input beams of the layer
  int I_node[64];
  double cum_p[64], cum_q[64];       // cumulative log-likelihoods of the input beams
  double lse_p[64], lse_q[64];       // fp64 log-sum-exp of their logit rows
  double max_p[64], max_q[64];       // exact row maxima
  double lm_p[64], lm_q[64];         // maxima of this workgroup's pieces of its rows (row i_lo first)
  float wmax[2][2 * VL_WAVES];       // per-wave maxima of a piece, two rows in flight
  double tmax[VL_BLOCK];             // partial row maxima of the gathering threads
  double sp[64], sq[64];             // beam weight / row sum: p_beam(i,x) = exp(z - max) * sp[i]
  double bw_p[64], bw_q[64];         // beam weights
  // accepted beams of the layer (next layer's inputs): node and its position among the candidates
  int A_node[64], A_idx[64];
  double A_cum_p[64], A_cum_q[64];
  // the prompt's nodes (loaded once: the sequential parts must not wait for global memory)
  int n_parent[NC], n_token[NC], n_rank[NC];
  short n_depth[NC];
  float n_u[NC];               // accept uniform of each node
  // candidates
  short slot_of[NC];           // slot in I of a prompt node, -1 if not an input beam
  int S_node[NC], S_tmp[NC];
  float S_zp[NC], S_zq[NC];   // logits at the candidates' (parent, token)
  double S_pb[NC], S_qb[NC];
  float S_u[NC];               // accept uniform of each candidate
  unsigned char S_flag[NC];    // test against p_beam itself: bit 0 = accepted, bit 1 = near tie
  // residual chain and accept-count table
  double cc[NC + 2], FF[NC + 2];
  union {
    struct { double alpha[NC + 2], first[NC + 2]; } w;   // dynamic width only
    double wpart[64 * VL_WAVES * 2];                                   // per-wave row sums of the exponential pass
  } u;
  double Pa[NC + 2], Pb[NC + 2];
  double wsum[2][VL_WAVES];
  unsigned long long acc_prev[2][NACC];   // the accumulator words' values before their next exchange
  double scan_w[VL_WAVES];
  double tsum[VL_BLOCK];
  double gpart[256];                 // one partial per workgroup of the prompt (G <= 256)
  double ptot[256];                  // p_beam total of every workgroup's slice, worked out from the layer's row sums
  int ptot_ok;                       // ... when every gathering thread saw a single piece (else 0: totals are exchanged)
  double exp_tab[64];                // 2^(j/64)
  double d_target[64];               // sampling: u * total of each draw
  // warped joints (top-k / top-p): union of the two supports, ascending flat index over I x V
  int U_idx[64];
  double U_p[64], U_q[64];
  int nU;
  double W_tau[2];                   // lower bounds of the slice's K-th entries
  int W_cnt[2];                      // entries kept per model after the merge
  int state[2];                      // outcome of the decision rounds, alternating entries
  int kmax, counter, abort, found, sbad, sgamma;
  int acc_n, pos, kidx;        // accept loop: accepted so far, next candidate, chain index of p'
  int pick_th;                 // sampling from workspace slices: the thread whose chunk holds the draw
};


static_assert(sizeof(LayerShared<NODE_CAP>) + VL_DYN_LDS_BYTES + 2048 <= CU_LDS_BYTES, "the layer kernel's LDS must fit a compute unit");
static_assert(sizeof(LayerShared<NODE_CAP_SMALL>) + VL_DYN_LDS_BYTES_SMALL + 2048 <= CU_LDS_BYTES, "the layer kernel's LDS must fit a compute unit");

// 2^(j/64), j = 0..63 (exp_nonpos.h)
__constant__ double c_exp2_tab[64] = {DSBD_EXP2_TABLE_64};

__device__ __forceinline__ double exp_nonpos(double x, const double* tab) { return dsbd_exp_nonpos(x, tab); }

// floor(a / b) for 0 <= a, 0 < b, both below 2^52, without the 64-bit integer division sequence
__device__ __forceinline__ long long div_floor(long long a, long long b) {
  long long q = (long long)((double)a / (double)b);
  if (q * b > a) --q;
  else if ((q + 1) * b <= a) ++q;
  return q;
}

// Wave-wide sum through the data-parallel-primitive lane moves (no LDS round trips as with shuffles): quads,
// rows of 16, then the row totals across the four rows; lane 63 ends up with the total, which is handed to every
// lane as a uniform value.  The order of the additions is fixed, so equal inputs give equal bits everywhere.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ double dpp_move_f64(double v) {       // lanes without a source lane read 0.0
  const int lo = __builtin_amdgcn_update_dpp(0, __double2loint(v), CTRL, ROW_MASK, 0xf, false);
  const int hi = __builtin_amdgcn_update_dpp(0, __double2hiint(v), CTRL, ROW_MASK, 0xf, false);
  return __hiloint2double(hi, lo);
}
template <int CTRL>
__device__ __forceinline__ unsigned long long dpp_move_u64(unsigned long long v) {
  const unsigned int lo = (unsigned int)__builtin_amdgcn_update_dpp(0, (int)(unsigned int)v, CTRL, 0xf, 0xf, false);
  const unsigned int hi = (unsigned int)__builtin_amdgcn_update_dpp(0, (int)(unsigned int)(v >> 32), CTRL, 0xf, 0xf, false);
  return ((unsigned long long)hi << 32) | lo;
}
__device__ __forceinline__ double wave_sum(double v) {
  v += dpp_move_f64<0xB1, 0xf>(v);    // quad_perm [1,0,3,2]
  v += dpp_move_f64<0x4E, 0xf>(v);    // quad_perm [2,3,0,1]
  v += dpp_move_f64<0x124, 0xf>(v);   // row_ror:4
  v += dpp_move_f64<0x128, 0xf>(v);   // row_ror:8: every lane holds the total of its row
  v += dpp_move_f64<0x142, 0xa>(v);   // row_bcast:15 into rows 1 and 3
  v += dpp_move_f64<0x143, 0xc>(v);   // row_bcast:31 into rows 2 and 3: lane 63 holds the total
  const int lo = __builtin_amdgcn_readlane(__double2loint(v), 63);
  const int hi = __builtin_amdgcn_readlane(__double2hiint(v), 63);
  return __hiloint2double(hi, lo);
}

// The largest of a value over the lanes of a wave, in every lane: rows of 16 by lane moves that pair the lanes
// symmetrically, the rows' results handed on to the rows behind, the last lane's read back as a uniform value.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_other_f32(float v) {          // lanes without a source lane read their own value
  return __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(v), __float_as_int(v), CTRL, ROW_MASK, 0xf, false));
}
__device__ __forceinline__ float wave_max_f32(float v) {
  v = fmaxf(v, dpp_other_f32<0xB1, 0xf>(v));    // quad_perm [1,0,3,2]
  v = fmaxf(v, dpp_other_f32<0x4E, 0xf>(v));    // quad_perm [2,3,0,1]
  v = fmaxf(v, dpp_other_f32<0x141, 0xf>(v));   // row_half_mirror
  v = fmaxf(v, dpp_other_f32<0x140, 0xf>(v));   // row_mirror
  v = fmaxf(v, dpp_other_f32<0x142, 0xa>(v));   // row_bcast:15 into rows 1 and 3
  v = fmaxf(v, dpp_other_f32<0x143, 0xc>(v));   // row_bcast:31 into rows 2 and 3
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}

// Inclusive prefix sums over the lanes of a wave by the same kind of lane moves: inside every row of 16 (sources
// outside the row count 0), then the row totals handed on to the rows behind.  Fixed order, equal bits everywhere.
__device__ __forceinline__ double wave_inclusive_scan(double v) {
  v += dpp_move_f64<0x111, 0xf>(v);   // row_shr:1
  v += dpp_move_f64<0x112, 0xf>(v);   // row_shr:2
  v += dpp_move_f64<0x114, 0xf>(v);   // row_shr:4
  v += dpp_move_f64<0x118, 0xf>(v);   // row_shr:8
  v += dpp_move_f64<0x142, 0xa>(v);   // row_bcast:15 into rows 1 and 3
  v += dpp_move_f64<0x143, 0xc>(v);   // row_bcast:31 into rows 2 and 3
  return v;
}
__device__ __forceinline__ double wave_max_all(double v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v = fmax(v, __shfl_xor(v, off));
  return v;
}

// Lanes of one wave handing values to each other through LDS: the hardware executes a wave's LDS instructions
// in order, but the compiler reasons per thread and would otherwise be free to reuse a value it loaded before
// another lane's store (or to forward only its own store).  This fence makes it reload.
__device__ __forceinline__ void wave_lds_fence() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Workgroup barrier that orders LDS traffic only.  __syncthreads() carries a workgroup-scope fence, for which the
// compiler also drains the wave's outstanding global loads and stores: where the waves exchange nothing but LDS
// values, this form lets the first wave's status stores and slot posts stay in flight across the barrier.
__device__ __forceinline__ void lds_barrier() {
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// Inclusive prefix sum over the block's threads in thread order (fixed tree: identical in every workgroup
// that scans the same values).
template <class Shared>
__device__ __forceinline__ double block_inclusive_scan(double v, Shared& sh) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  v = wave_inclusive_scan(v);
  __syncthreads();
  if (lane == 63) sh.scan_w[wave] = v;
  __syncthreads();
  double before = 0.0;
  for (int w = 0; w < wave; ++w) before += sh.scan_w[w];
  return before + v;
}

// ---- exchange among the G workgroups of one prompt
//
// No grid-wide barrier and no cache-wide fence: a workgroup publishes each partial value in its own
// 16-byte slot as two agent-scope atomic words (value bits, value bits XOR tag) and every other
// workgroup polls exactly the slots it needs.  The tag changes with every exchange, so a slot is valid
// only once both words of the current exchange have landed.  A bank of slots is never overwritten while
// somebody may still read it:
//  * exchanges that every workgroup posts and then collects at once from all the others (chain entries,
//    sampling prefixes, warping candidates) alternate between banks 0 and 1: whoever posts exchange n + 2 has
//    collected n + 1, so everybody had posted n + 1 and was therefore done collecting n;
//  * the row-sum exchange (collected only from the workgroups that share a row) and the early post of the
//    chain's second entry (collected later, or never) give no such guarantee, so each layer has a bank of its
//    own for either of them, written once per launch;
//  * the three hops of the warping merge (every workgroup -> its group's first -> the prompt's first -> every
//    workgroup) have a bank each: nobody posts a hop of the next layer before having received the result of
//    this one, which exists only after every reader of the earlier hops is done.
struct Slot { unsigned long long w0, w1; };

__device__ __forceinline__ unsigned long long exchange_tag(unsigned long long epoch) {
  return epoch * 0x9E3779B97F4A7C15ull;
}

__device__ __forceinline__ void slot_post(Slot* s, double v, unsigned long long tag) {
  const unsigned long long b = (unsigned long long)__double_as_longlong(v);
  __hip_atomic_store(&s->w0, b, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  __hip_atomic_store(&s->w1, b ^ tag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Waits until the slot carries the tag; gives up after `limit` ticks of the wall clock (returns false).
__device__ __forceinline__ bool slot_wait(Slot* s, unsigned long long tag, double& v, long long limit) {
  long long t0 = 0;
  for (int spin = 0;; ++spin) {
    const unsigned long long w0 = __hip_atomic_load(&s->w0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const unsigned long long w1 = __hip_atomic_load(&s->w1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if ((w0 ^ w1) == tag) { v = __longlong_as_double((long long)w0); return true; }
    if (spin == 0) t0 = wall_clock64();
    else if ((spin & 15) == 0 && wall_clock64() - t0 > limit) return false;
    __builtin_amdgcn_s_sleep(1);
  }
}

// The same for two slots at once (their loads in flight together).
__device__ __forceinline__ bool slot_wait2(Slot* s0, Slot* s1, unsigned long long tag, double& v0, double& v1, long long limit) {
  long long t0 = 0;
  bool h0 = false, h1 = false;
  for (int spin = 0;; ++spin) {
    unsigned long long a0 = 0, a1 = 0, b0 = 0, b1 = 0;
    if (!h0) { a0 = __hip_atomic_load(&s0->w0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); a1 = __hip_atomic_load(&s0->w1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
    if (!h1) { b0 = __hip_atomic_load(&s1->w0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); b1 = __hip_atomic_load(&s1->w1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
    if (!h0 && (a0 ^ a1) == tag) { v0 = __longlong_as_double((long long)a0); h0 = true; }
    if (!h1 && (b0 ^ b1) == tag) { v1 = __longlong_as_double((long long)b0); h1 = true; }
    if (h0 && h1) return true;
    if (spin == 0) t0 = wall_clock64();
    else if ((spin & 15) == 0 && wall_clock64() - t0 > limit) return false;
    __builtin_amdgcn_s_sleep(1);
  }
}

// Single-value exchanges: workgroup w owns the slot at the start of its own 128-byte line of the bank (slot index
// w * LINE_SLOTS), so that no two workgroups ever write the same cache line.  Measured with a microbenchmark
// on this chip, all-to-all among 256 workgroups: 2.3 us with a line per workgroup, 3.1 us with the words packed
// densely (sixteen writers per line), although the packed layout needs sixteen times fewer lines per poll.
#define LINE_SLOTS 8
__device__ __forceinline__ void dense_post(Slot* bank, int G, int g, double v, unsigned long long tag) {
  (void)G;
  slot_post(bank + (long long)g * LINE_SLOTS, v, tag);
}

// One wave collects the values of all G workgroups (G <= 256): lane i gets those of workgroups i, i + 64, i + 128,
// i + 192 in v[0..3] (0 beyond G), with the loads of a polling round in flight together; `own` is the value this
// workgroup posted.  False if the wait gave up.
__device__ __forceinline__ bool wave_collect4(Slot* bank, int G, int g, double own, unsigned long long tag,
                                              double (&v)[4], long long limit) {
  const int lane = threadIdx.x & 63;
  bool have[4];
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    have[k] = (lane + 64 * k >= G); v[k] = 0.0;
    if (lane + 64 * k == g) { have[k] = true; v[k] = own; }   // the workgroup's own value needs no round trip
  }
  long long t0 = 0;
  for (int spin = 0;; ++spin) {
    unsigned long long w0[4], w1[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      w0[k] = 0; w1[k] = 0;
      if (!have[k]) {
        Slot* s = bank + (long long)(lane + 64 * k) * LINE_SLOTS;
        w0[k] = __hip_atomic_load(&s->w0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        w1[k] = __hip_atomic_load(&s->w1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
    }
#pragma unroll
    for (int k = 0; k < 4; ++k)
      if (!have[k] && (w0[k] ^ w1[k]) == tag) { v[k] = __longlong_as_double((long long)w0[k]); have[k] = true; }
    if (have[0] && have[1] && have[2] && have[3]) return true;
    if (spin == 0) t0 = wall_clock64();
    else if ((spin & 15) == 0 && wall_clock64() - t0 > limit) return false;
    __builtin_amdgcn_s_sleep(1);
  }
}

// Sum over the prompt's G workgroups of one value each, for the first wave of every workgroup; the value is already
// posted (or being posted) in the workgroup's line of `bank`.  With more than SUM_GROUP workgroups the sum takes two
// hops: the first workgroup of every group of SUM_GROUP adds up its group's values and posts the group sum in
// `gbank`, and everybody adds up the at most SUM_GROUPS group sums.  Each workgroup then polls 16 + 16 lines instead
// of 256, and all of them add the same numbers in the same order.  False if a wait gave up.
#define SUM_GROUP 16
#define SUM_GROUPS 16
__device__ __forceinline__ bool wave_sum_groups(Slot* bank, Slot* gbank, int G, int g, double own,
                                                unsigned long long tag, long long limit, double& total) {
  const int lane = threadIdx.x & 63;
  if (G <= SUM_GROUP) {
    double v[4];
    const bool ok = wave_collect4(bank, G, g, own, tag, v, limit);
    total = wave_sum((v[0] + v[1]) + (v[2] + v[3]));
    return ok;
  }
  bool ok = true;
  const int first = g - g % SUM_GROUP, n_groups = (G + SUM_GROUP - 1) / SUM_GROUP;
  double gs_own = 0.0;
  if (g == first) {
    const int n_mem = min(SUM_GROUP, G - first);
    double v = 0.0;
    if (lane == 0) v = own;
    else if (lane < n_mem) ok = slot_wait(bank + (long long)(first + lane) * LINE_SLOTS, tag, v, limit);
    gs_own = wave_sum(v);
    if (lane == 0) slot_post(gbank + (long long)(g / SUM_GROUP) * LINE_SLOTS, gs_own, tag);
  }
  double c = 0.0;
  if (lane < n_groups) {
    if (g == first && lane == g / SUM_GROUP) c = gs_own;          // the workgroup's own group sum needs no round trip
    else ok = slot_wait(gbank + (long long)lane * LINE_SLOTS, tag, c, limit) && ok;
  }
  total = wave_sum(c);
  return __builtin_amdgcn_ballot_w64(!ok) == 0ull;
}

// Sum over the prompt's G workgroups of one value in [0, 4) each, in one hop: every workgroup adds its value, as a
// 2^-52 fixed-point number with a 1 in the count field above it, to one of NACC accumulator words (an agent-scope
// integer atomic: the order of the additions does not matter, so the sum is the same in every run), and one wave
// polls the NACC words until each has counted all its members.  The accumulators are never cleared: a word only ever
// grows (modulo 2^64), and what an exchange added to it is the difference to the value it had before the exchange,
// which every workgroup knows (the value it read at the end of the word's previous exchange; the values at launch are
// read by the prompt's first workgroup before anybody adds and handed round with the first layer's row sums).  The
// difference decodes as (members << 54) + sum as long as the sum stays below 2^54 units and there are fewer than 1024
// members per word.  Two banks alternate as for the slot exchanges.  Measured among 256 workgroups: 1.8 us against
// 2.45 us for the two-hop slot exchange (a microbenchmark of both on the same box).
__device__ __forceinline__ bool wave_sum_accumulators(unsigned long long* accs, unsigned long long* prev, int G, int g,
                                                      double own, long long limit, double& total) {
  const int lane = threadIdx.x & 63;
  if (G == 1) { total = own; return true; }
  if (lane == 0) {
    const unsigned long long q = (unsigned long long)__double2ull_rn(fmin(fmax(own, 0.0), 3.999) * 4503599627370496.0);
    __hip_atomic_fetch_add(&accs[(g % NACC) * 16], (1ull << ACC_FIELD_BITS) + q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  bool ok = true;
  unsigned long long field = 0;
  if (lane < NACC) {
    const unsigned long long members = lane < G ? (unsigned long long)((G - lane + NACC - 1) / NACC) : 0ull;
    if (members) {
      const unsigned long long before = prev[lane];
      long long t0 = 0;
      for (int spin = 0;; ++spin) {
        const unsigned long long w = __hip_atomic_load(&accs[lane * 16], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const unsigned long long diff = w - before;
        if ((diff >> ACC_FIELD_BITS) == members) { field = diff & ((1ull << ACC_FIELD_BITS) - 1); prev[lane] = w; break; }
        if (spin == 0) t0 = wall_clock64();
        else if ((spin & 15) == 0 && wall_clock64() - t0 > limit) { ok = false; break; }
        __builtin_amdgcn_s_sleep(1);
      }
    }
  }
  // the eight words' fields added up by lane moves inside the SIMD (quads, then the other quad of the eight) and the
  // first lane's total read back as a uniform value: no LDS round trips on the chain's critical path
  static_assert(NACC == 8, "the reduction below is written for eight words");
  field += dpp_move_u64<0xB1>(field);       // quad_perm [1,0,3,2]
  field += dpp_move_u64<0x4E>(field);       // quad_perm [2,3,0,1]
  field += dpp_move_u64<0x141>(field);      // row_half_mirror
  {
    const unsigned int lo = (unsigned int)__builtin_amdgcn_readfirstlane((int)(unsigned int)field);
    const unsigned int hi = (unsigned int)__builtin_amdgcn_readfirstlane((int)(unsigned int)(field >> 32));
    field = ((unsigned long long)hi << 32) | lo;
  }
  total = (double)field * (1.0 / 4503599627370496.0);
  return __builtin_amdgcn_ballot_w64(!ok) == 0ull;
}

__device__ __forceinline__ Slot* prompt_slots(const LayersArgs& a, int prompt) {
  return reinterpret_cast<Slot*>(a.red) + (long long)prompt * a.sl.prompt_stride;
}

// ---- selection of the largest joint entries (warping T).  Entries are ranked by descending value, equal values by
// ascending flat index; a candidate is (value, index), "none" is (-1, INT_MAX).
#define WARP_K_MAX 32
#define WARP_CAND 512          // candidates per model a merge can hold (WARP_GROUP lists of WARP_K_MAX entries)
#define WARP_GROUP 16          // workgroups whose lists one workgroup merges
__device__ __forceinline__ bool cand_before(double va, int ia, double vb, int ib) {
  // no short circuit: the operands are loaded side by side instead of one after a branch on the other
  return (va > vb) | ((va == vb) & (ia < ib));
}
__device__ __forceinline__ double readlane_f64(double v, int l) {
  const int lo = __builtin_amdgcn_readlane(__double2loint(v), l), hi = __builtin_amdgcn_readlane(__double2hiint(v), l);
  return __hiloint2double(hi, lo);
}
// first candidate in rank order among one per lane; the same result in every lane
__device__ __forceinline__ void wave_first(double& v, int& i) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    const double ov = __shfl_xor(v, off);
    const int oi = __shfl_xor(i, off);
    if (cand_before(ov, oi, v, i)) { v = ov; i = oi; }
  }
}

// How a layer's joint over nI rows of V entries is cut among G workgroups (host and device use the same rule).
struct SliceCut {
  int rows_per_wg;       // > 0: every workgroup takes this many whole rows (nI >= G)
  int wg_per_row;        // else: every row is cut into this many pieces of `len` entries (the last ones may be empty)
  long long len;         // entries of the longest slice
};
__host__ __device__ inline SliceCut slice_cut(int nI, int V, int G) {
  SliceCut c;
  if (nI >= G) {
    c.rows_per_wg = (nI + G - 1) / G; c.wg_per_row = 0; c.len = (long long)c.rows_per_wg * V;
  } else {
    c.rows_per_wg = 0; c.wg_per_row = G / nI;
    c.len = (((long long)V + c.wg_per_row - 1) / c.wg_per_row + 1) & ~1LL;
  }
  return c;
}

// At most VL_MAX_VGPRS vector registers, so that a wave of the statistics pass (32 registers) fits on every SIMD beside
// this kernel's two: 2 x 240 + 32 = 512.  (The attribute counts in halves of the unified register file of this
// target: the compiler doubles the number it is given.  Without it the allocator takes whatever two waves per SIMD
// leave it, up to 256, whether it needs them or not.)
#define VL_MAX_VGPRS 240
template <bool WARP, int NC>
__global__ __launch_bounds__(VL_BLOCK) __attribute__((amdgpu_num_vgpr(VL_MAX_VGPRS / 2)))
void verify_layers_kernel(LayersArgs a) {
  __shared__ LayerShared<NC> sh;
  extern __shared__ __attribute__((aligned(16))) double dyn_lds[];
  const int prompt = a.prompt0 + blockIdx.x / a.G;
  const int g = blockIdx.x % a.G;
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int V = a.V;
  unsigned int epoch = 0;      // exchanges so far (sets the tag); identical in every workgroup of the prompt
  unsigned int xchg = 0;       // of those, the ones on the two alternating banks
  Slot* const slots = prompt_slots(a, prompt);
  // (a replayed launch: the replay count, which the kernel in front of this one has just raised, sets the tags apart
  // from those of the graph's earlier replays)
  const unsigned long long nonce =
      a.nonce + (a.replay ? (__hip_atomic_load(a.replay, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) << 40) : 0ull);
  // (selected, not indexed: a run-time index into the kernel's argument block would move the whole block into scratch memory)
  const int slx0 = a.sl.x[0], slx1 = a.sl.x[1], slxc0 = a.sl.xc[0], slxc1 = a.sl.xc[1];
  auto bank_x = [&](unsigned int n) { return (n & 1) ? slx1 : slx0; };
  auto bank_xc = [&](unsigned int n) { return (n & 1) ? slxc1 : slxc0; };
  unsigned int wsum_round = 0; // alternates the two wsum buffers
  unsigned int decide_round = 0;
  int trace_n = 0;
  auto stamp = [&](int label) {
    if (a.trace && (int)blockIdx.x == a.trace_wg && tid == 0 && trace_n < 255) {
      a.trace[2 * trace_n + 2] = label; a.trace[2 * trace_n + 3] = wall_clock64(); ++trace_n; a.trace[0] = trace_n;
    }
  };
  stamp(0);

  // the accumulator words of the one-hop sums as the launch finds them: read by the prompt's first workgroup before
  // anybody adds to them (nobody does before the first layer's row sums, which wait for this workgroup's), and handed
  // to the others in tagged slots, collected during the first layer
  unsigned long long* const accs = reinterpret_cast<unsigned long long*>(slots + a.sl.acc);
  const unsigned long long acc0_tag = exchange_tag(nonce + 0xFFFFFFull);
  unsigned int achg = 0;       // accumulator exchanges so far (alternates their two banks)
  // (requested here, used at the end of the prologue: the round trip through the memory system runs beside it)
  unsigned long long acc0_w = 0;
  if (g == 0 && tid < 2 * NACC)
    acc0_w = __hip_atomic_load(&accs[tid * 16], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);

  if (tid == 0) { sh.abort = 0; sh.sbad = 0; sh.sgamma = 0; sh.counter = 0; sh.found = 0; }
  double exp_tab_mine = 0.0;     // (the table entry travels while the prompt's trees are looked up; stored below)
  if (tid < 64) exp_tab_mine = c_exp2_tab[tid];

  // ---- trees and nodes of this prompt.  tree_prompt is non-decreasing: the prompt's trees are those behind the
  // trees of earlier prompts.  (Everything the kernel needs it derives from the call's inputs: it does not wait for
  // the statistics pass, which runs beside it.)
  int t_first = 0, t_end = a.n_trees;
  if (a.n_prompts > 1) {
    __syncthreads();
    int lt = 0, le = 0;
    for (int t = tid; t < a.n_trees; t += VL_BLOCK) {
      const int tp = a.tree_prompt[t];
      lt += tp < prompt; le += tp <= prompt;
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) { lt += __shfl_xor(lt, off); le += __shfl_xor(le, off); }
    if (lane == 0) { atomicAdd(&sh.counter, lt); atomicAdd(&sh.found, le); }
    __syncthreads();
    t_first = sh.counter; t_end = sh.found;
  }
  stamp(2);
  int n_roots = t_end - t_first;
  int bad = 0;
  if (n_roots < 0) { bad |= DSBD_FAULT_TOPOLOGY; n_roots = 0; }
  if (n_roots > a.max_prompt_trees || n_roots > a.I_cap || n_roots > 64) { bad |= DSBD_FAULT_BOUNDS; n_roots = 0; }
  int n_begin = 0, n_end = 0;
  if (n_roots > 0) { n_begin = a.tree_off[t_first]; n_end = a.tree_off[t_end]; }
  if (n_begin < 0 || n_end > a.n_nodes || n_end < n_begin) { bad |= DSBD_FAULT_TOPOLOGY; n_roots = 0; }
  if (n_end - n_begin > NC) { bad |= DSBD_FAULT_BOUNDS; n_roots = 0; }
  int n_pn = n_roots > 0 ? n_end - n_begin : 0;          // nodes of the prompt
  const int Lw = a.max_depth + 2;                        // row length of the per-layer arrays
  stamp(3);
  __syncthreads();
  if (tid < n_roots) {                                   // every tree inside the prompt's node range
    const int b = t_first + tid;
    const int r0 = a.tree_off[b], r1 = a.tree_off[b + 1];
    if (r0 < n_begin || r1 > n_end || r1 <= r0) atomicOr(&sh.sbad, DSBD_FAULT_TOPOLOGY);
    sh.I_node[tid] = r0;
    sh.cum_p[tid] = a.blp[b];
    sh.cum_q[tid] = a.blq[b];
  }
  if (tid < n_pn) {
    const int n = n_begin + tid;
    int tok = a.token[n];
    if (tok < 0 || tok >= V) { atomicOr(&sh.sbad, DSBD_FAULT_TOKEN); tok = 0; }
    sh.n_parent[tid] = a.parent[n];
    sh.n_token[tid] = tok;
    sh.n_rank[tid] = a.rank ? a.rank[n] : 0;
    sh.n_u[tid] = a.u_acc[n];
    sh.slot_of[tid] = -1;
    sh.S_tmp[tid] = 0;
  }
  if (tid < 64) sh.exp_tab[tid] = exp_tab_mine;
  __syncthreads();
  stamp(4);
  if (sh.sbad & DSBD_FAULT_TOPOLOGY) { n_roots = 0; n_pn = 0; }
  // node depths (and the validation of the parent pointers): one wave per tree walks the parent chains with lane
  // shuffles over the entries already in the LDS; depths land in S_tmp (prompt-local index)
  for (int b = wave; b < n_roots; b += VL_WAVES) {
    dsbd_tree_range t;
    t.base = sh.I_node[b];
    t.n_all = (b + 1 < n_roots ? sh.I_node[b + 1] : n_end) - t.base;
    t.n = min(t.n_all, min(a.max_tree_nodes, DSBD_MAX_TREE_NODES));
    t.bad = t.n_all > t.n ? DSBD_FAULT_BOUNDS : 0;
    t.valid = true;
    const int p_mine = lane < t.n ? sh.n_parent[t.base - n_begin + lane] : -1;
    const int fb = dsbd_tree_walk(t, lane, p_mine, a.max_depth, reinterpret_cast<int32_t*>(sh.S_tmp) - n_begin, nullptr, nullptr);
    if (fb) atomicOr(&sh.sbad, fb);
    // the tree's deepest node: the wave's maximum by lane exchanges, one LDS atomic per tree (an atomic per node, all
    // on one word, took 2 us on a prompt of 248 nodes)
    wave_lds_fence();
    const int d_mine = lane < t.n ? sh.S_tmp[t.base - n_begin + lane] : 0;
    int d = d_mine;
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) d = max(d, __shfl_xor(d, off));
    if (lane == 0 && d > 0) atomicMax(&sh.sgamma, d);
    // (the node's tree within the prompt rides in the bits above its depth: the next-beam plan names it)
    if (lane < t.n) sh.S_tmp[t.base - n_begin + lane] = (d_mine & NODE_DEPTH_MASK) | (b << NODE_TREE_SHIFT);
  }
  __syncthreads();
  if (tid < n_pn) sh.n_depth[tid] = (short)sh.S_tmp[tid];      // (read after later barriers only)
  stamp(5);
  bad |= sh.sbad;
  const int gamma = min(sh.sgamma, a.max_depth);
  if (bad && g == 0 && tid == 0) atomicOr(a.fault, bad);

  // ---- initial statuses (first workgroup of the prompt)
  if (g == 0) {
    if (tid < n_pn) a.out.node_status[n_begin + tid] = (sh.n_depth[tid] & NODE_DEPTH_MASK) == 0 ? DSBD_ROOT : DSBD_NOT_REACHED;
    for (int i = tid; i < Lw; i += VL_BLOCK) a.out.layer_width[(long long)prompt * Lw + i] = i == 0 ? n_roots : 0;
  }
  // Output words are written by exactly one workgroup each (sampled beams by the workgroup that owns the
  // sample, per-node log-probabilities by the node's workgroup, everything else by the prompt's first
  // workgroup): the XCDs' L2 caches are not coherent with each other, so two workgroups must never write
  // the same word.
  const int plan_len = a.max_depth + 1;                   // row length of the plan's paths
  auto clear_out_slots = [&](int from) {
    for (int i = from + tid; i < a.W_cap; i += VL_BLOCK) {
      const long long o = (long long)prompt * a.W_cap + i;
      a.out.out_parent[o] = -1; a.out.out_token[o] = -1; a.out.out_node[o] = -1;
      a.out.out_logp_target[o] = 0.0; a.out.out_logp_draft[o] = 0.0;
      if (a.nx_on) {
        a.nx.src_tree[o] = -1; a.nx.src_out[o] = -1; a.nx.path_len[o] = 0; a.nx.token[o] = -1;
        a.nx.logp_target[o] = 0.0; a.nx.logp_draft[o] = 0.0;
        for (int k = 0; k < plan_len; ++k) a.nx.path[o * plan_len + k] = -1;
      }
    }
  };
  // Fused selection (Algorithm 1's return; Section 3.3, last paragraph): whoever writes output beam j of the prompt
  // also writes its entry of the next-beam plan: the tree whose cache it continues and the nodes root .. `node`
  // (the beam's last forest node), root first, read off the parent entries in the LDS.  One thread per beam.
  auto emit_next = [&](int j, int node, int x, double lp, double lq) {
    if (!a.nx_on) return;
    const long long o = (long long)prompt * a.W_cap + j;
    const int dt = sh.n_depth[node - n_begin];
    const int d = min(dt & NODE_DEPTH_MASK, a.max_depth);
    int32_t* const path = a.nx.path + o * plan_len;
    int cur = node;
    for (int k = d; k >= 0; --k) {
      path[k] = cur;
      cur = k > 0 ? sh.n_parent[cur - n_begin] : cur;
    }
    for (int k = d + 1; k < plan_len; ++k) path[k] = -1;
    a.nx.src_tree[o] = t_first + (dt >> NODE_TREE_SHIFT);
    a.nx.src_out[o] = j;
    a.nx.path_len[o] = d + 1;
    a.nx.token[o] = x;
    a.nx.logp_target[o] = lp;
    a.nx.logp_draft[o] = lq;
  };
  if (n_roots == 0) {
    if (g == 0) clear_out_slots(0);
    if (g == 0 && tid == 0) {
      a.out.l_last[prompt] = 0; a.out.n_out[prompt] = 0; a.out.near_tie_count[prompt] = 0;
      if (a.nx_on) a.nx.n_next[prompt] = 0;
    }
    return;   // uniform over the prompt's workgroups: nobody waits for a missing partner
  }

  const int W_in = a.W_L > 0 ? a.W_L : n_roots;
  const bool dynamic = a.t >= 0.f;
  const double thr = (double)a.t;
  // Slices that do not fit the LDS live in the workspace, each workgroup's in a region of its own: the layers
  // cut I x V differently, and an address written by workgroups of two XCDs in turn (whose L2 caches write back
  // in no particular order) could later be read back stale.
  double* pb = a.pb + (long long)blockIdx.x * a.slice_cap;
  double* qb = a.qb + (long long)blockIdx.x * a.slice_cap;
  const float* u_res = a.u_res + (long long)prompt * Lw;
  const float* u_fill = a.u_fill + (long long)prompt * Lw * a.W_cap;

  // ---- layer 1 inputs: the roots
  if (tid < n_roots) sh.slot_of[sh.I_node[tid] - n_begin] = (short)tid;
  int nI = n_roots;
  int near_tie = 0;          // meaningful in thread 0
  int l_last = gamma + 1;
  int n_out = 0;
  if (g == 0 && tid < 2 * NACC) {
    (&sh.acc_prev[0][0])[tid] = acc0_w;
    slot_post(slots + a.sl.acc0 + tid, __longlong_as_double((long long)acc0_w), acc0_tag);
  }
  __syncthreads();
  stamp(6);

  // total over the workgroup of one value per thread: valid in every thread after the barrier inside
  auto wg_total = [&](double s, bool lds_only = false) -> double {
    s = wave_sum(s);
    double* ws = sh.wsum[wsum_round & 1];
    wsum_round += 1;
    if (lane == 0) ws[wave] = s;
    if (lds_only) lds_barrier(); else __syncthreads();
    return ((ws[0] + ws[1]) + (ws[2] + ws[3])) + ((ws[4] + ws[5]) + (ws[6] + ws[7]));
  };
  auto give_up = [&]() { sh.abort = 1; atomicOr(a.fault, DSBD_FAULT_SYNC_TIMEOUT); };

  // this workgroup's share of I x V, as a function of the number of rows
  int geo_nI = -1, geo_ilo = 0, geo_ihi = -1, geo_pieces = 1;
  SliceCut geo_cut = {0, 1, 0};
  long long geo_lo = 0, geo_hi = 0;

  // (worked out when the number of rows changes: a handful of 64-bit divisions, on every workgroup's critical
  // path, that a fixed layer width repeats unchanged layer after layer)
  auto set_geometry = [&](int rows) {
    if (rows == geo_nI) return;
    const long long all = (long long)rows * V;
    geo_nI = rows;
    geo_cut = slice_cut(rows, V, a.G);
    geo_lo = all; geo_hi = all;
    if (geo_cut.rows_per_wg > 0) {
      geo_lo = min(all, (long long)g * geo_cut.rows_per_wg * V);
      geo_hi = min(all, geo_lo + (long long)geo_cut.rows_per_wg * V);
    } else if (g / geo_cut.wg_per_row < rows) {
      const long long r0 = (long long)(g / geo_cut.wg_per_row) * V, k = g % geo_cut.wg_per_row;
      geo_lo = r0 + min((long long)V, k * geo_cut.len);
      geo_hi = r0 + min((long long)V, (k + 1) * geo_cut.len);
    }
    geo_ilo = (int)div_floor(geo_lo, V);
    geo_ihi = geo_hi > geo_lo ? (int)div_floor(geo_hi - 1, V) : geo_ilo - 1;
    geo_pieces = (int)((V + geo_cut.len - 1) / geo_cut.len);
  };
  int passed_nacc = -1;      // >= 0: the layer before passed with this many accepted beams, not yet handed over

  stamp(1);
  for (int l = 1; l <= gamma + 1; ++l) {
    stamp(10 + l);
    // The layer before passed: its accepted beams are this layer's inputs.  The first two rounds of logits of this
    // workgroup's first row are requested BEFORE the hand-over's book-keeping, which then runs while they travel
    // (its barriers order the LDS only).
    float eA_p[XU], eA_q[XU], eB_p[XU], eB_q[XU];
    bool early = false;
#pragma unroll
    for (int k = 0; k < XU; ++k) { eA_p[k] = 0.f; eA_q[k] = 0.f; eB_p[k] = 0.f; eB_q[k] = 0.f; }
    if (passed_nacc >= 0) {
      const int nacc = passed_nacc;
      passed_nacc = -1;
      set_geometry(nacc);
      if (geo_ihi >= geo_ilo) {
        const int i = geo_ilo;
        const int node = sh.A_node[i];
        const int x_lo = (int)(max(geo_lo, (long long)i * V) - (long long)i * V);
        const int x_hi = (int)(min(geo_hi, (long long)(i + 1) * V) - (long long)i * V);
        const float* zp = a.zp + (long long)node * V;
        const float* zq = a.zq + (long long)node * V;
        const int xA = x_lo + tid, xB = xA + XU * VL_BLOCK;
#pragma unroll
        for (int k = 0; k < XU; ++k) {
          const int xx = min(xA + k * VL_BLOCK, x_hi - 1);
          eA_p[k] = zp[xx]; eA_q[k] = zq[xx];
        }
#pragma unroll
        for (int k = 0; k < XU; ++k) {
          const int xx = min(xB + k * VL_BLOCK, x_hi - 1);
          eB_p[k] = zp[xx]; eB_q[k] = zq[xx];
        }
        early = true;
      }
      // cumulative likelihoods of the accepted beams (fp64)
      if (tid < nacc) {
        const int n = sh.A_node[tid];
        const int ci = sh.A_idx[tid];
        const int slot = sh.slot_of[sh.n_parent[n - n_begin] - n_begin];
        sh.A_cum_p[tid] = sh.cum_p[slot] + ((double)sh.S_zp[ci] - sh.lse_p[slot]);
        sh.A_cum_q[tid] = sh.cum_q[slot] + ((double)sh.S_zq[ci] - sh.lse_q[slot]);
      }
      lds_barrier();
      // (no barrier between the next two steps: the old inputs and the new ones are nodes of different depths, so
      // their slot_of entries are different words, and thread t reads I_node[t] before it alone overwrites it)
      if (tid < nI) sh.slot_of[sh.I_node[tid] - n_begin] = -1;
      if (tid < nacc) {
        const int i = sh.A_node[tid] - n_begin;
        sh.I_node[tid] = sh.A_node[tid];
        sh.cum_p[tid] = sh.A_cum_p[tid];
        sh.cum_q[tid] = sh.A_cum_q[tid];
        sh.slot_of[i] = (short)tid;
      }
      nI = nacc;
      lds_barrier();
    }
    const bool bonus = (l == gamma + 1);
    const long long total = (long long)nI * V;           // elements of I x V
    // I x V is cut along the rows: with fewer rows than workgroups every row is cut into the same pieces (the
    // workgroups left over idle for the layer), otherwise every workgroup takes whole rows.  Either way a row's
    // sum is formed in an order that depends on the row's length only, so beams with equal logits and equal
    // likelihoods (duplicates are common in beam sampling) get bitwise equal joint entries, and the order of
    // equal entries (by index) is the same as in a plain row-by-row evaluation.
    set_geometry(nI);
    const SliceCut cut = geo_cut;
    const long long ch = cut.len;            // the longest slice of the layer
    const long long e_lo = geo_lo, e_hi = geo_hi;
    const long long len = e_hi - e_lo;
    const int i_lo = geo_ilo, i_hi = geo_ihi;
    // slice storage: the leading n_lds entries of the slice in the LDS (no memory latency in the dependent passes, and
    // no traffic: a batch of prompts whose slices all lived in the workspace re-read them through the memory system
    // a dozen times per layer), what does not fit behind them in the workspace
    const long long n_lds = min(len, (long long)a.lds_slice);
    const bool in_lds = n_lds == len;
    // Accessors with explicit address spaces (LDS or global): through generic pointers the compiler merges the two
    // cases into one FLAT access with a selected address, which is slower than either.
    typedef __attribute__((address_space(3))) double lds_f64;
    typedef __attribute__((address_space(1))) double glb_f64;
    lds_f64* const pl = (lds_f64*)dyn_lds;
    lds_f64* const ql = a.alias ? pl : pl + a.lds_elems;
    glb_f64* const pbg = (glb_f64*)pb;
    glb_f64* const qbg = a.alias ? pbg : (glb_f64*)qb;
    auto ldp = [&](long long j) -> double { double v; if (j < n_lds) v = pl[(int)j]; else v = pbg[j]; return v; };
    auto ldq = [&](long long j) -> double { double v; if (j < n_lds) v = ql[(int)j]; else v = qbg[j]; return v; };
    // The hot loops are written once, over a range [r0, r1) of the slice, and instantiated for both homes, with the
    // choice taken outside the loop (left per access, it becomes a pair of branches around every load and store).
    auto with_slices = [&](auto&& body) __attribute__((always_inline)) {
      if (in_lds) { body(pl, ql, 0LL, len); return; }
      if (n_lds > 0) body(pl, ql, 0LL, n_lds);
      body(pbg, qbg, n_lds, len);
    };

    // ===== p_beam / q_beam over I x V: exponentials and this workgroup's share of the row sums.  The exponentials
    // are taken against the maximum of the workgroup's own piece of the row (found here, in the same pass over the
    // logits); the pieces' maxima travel with their sums and are folded into the row's maximum and total below.
    for (int i = i_lo; i <= i_hi; ++i) {
      const int node = sh.I_node[i];
      const int x_lo = (int)(max(e_lo, (long long)i * V) - (long long)i * V);      // positions in the row: below V < 2^30
      const int x_hi = (int)(min(e_hi, (long long)(i + 1) * V) - (long long)i * V);
      const float* zp = a.zp + (long long)node * V;
      const float* zq = a.zq + (long long)node * V;
      double s_p = 0.0, s_q = 0.0;
      const long long joff = (long long)i * V - e_lo;
      auto exp_pass = [&](auto store) __attribute__((always_inline)) {
      // the first two rounds of XU logits per model stay in registers (a 4008-entry piece of the benchmark's joint is
      // two rounds); longer pieces are read a second time (from the caches)
      float fpA[XU], fqA[XU], fpB[XU], fqB[XU];
      float lmp = -INFINITY, lmq = -INFINITY;
      const int xA = x_lo + tid, xB = xA + XU * VL_BLOCK;
      const bool haveB = x_lo + XU * VL_BLOCK < x_hi;                      // uniform over the workgroup
      if (early && i == i_lo) {            // requested at the top of the layer
#pragma unroll
        for (int k = 0; k < XU; ++k) { fpA[k] = eA_p[k]; fqA[k] = eA_q[k]; fpB[k] = eB_p[k]; fqB[k] = eB_q[k]; }
      } else {
#pragma unroll
        for (int k = 0; k < XU; ++k) {
          const int xx = min(xA + k * VL_BLOCK, x_hi - 1);              // clamped repeats do not change a maximum
          fpA[k] = zp[xx]; fqA[k] = zq[xx];
        }
#pragma unroll
        for (int k = 0; k < XU; ++k) {
          const int xx = min(xB + k * VL_BLOCK, x_hi - 1);
          fpB[k] = zp[xx]; fqB[k] = zq[xx];
        }
      }
      bool nonfinite = false;        // (the statistics pass reports these for every row; this kernel for the rows it uses)
#pragma unroll
      for (int k = 0; k < XU; ++k) {
        lmp = fmaxf(fmaxf(lmp, fpA[k]), fpB[k]); lmq = fmaxf(fmaxf(lmq, fqA[k]), fqB[k]);
        nonfinite |= !(fpA[k] <= FLT_MAX) | !(fqA[k] <= FLT_MAX) | !(fpB[k] <= FLT_MAX) | !(fqB[k] <= FLT_MAX);     // NaN or +Inf (-Inf: a masked token)
      }
      // (the rest of a long piece: maxima only, so four times as many logits in flight as in the rounds above)
      for (int x = xB + XU * VL_BLOCK; x < x_hi; x += 4 * XU * VL_BLOCK) {
        float fp[4 * XU], fq[4 * XU];
#pragma unroll
        for (int k = 0; k < 4 * XU; ++k) {
          const int xx = min(x + k * VL_BLOCK, x_hi - 1);
          fp[k] = zp[xx]; fq[k] = zq[xx];
        }
#pragma unroll
        for (int k = 0; k < 4 * XU; ++k) {
          lmp = fmaxf(lmp, fp[k]); lmq = fmaxf(lmq, fq[k]);
          nonfinite |= !(fp[k] <= FLT_MAX) | !(fq[k] <= FLT_MAX);
        }
      }
      if (nonfinite) atomicOr(a.fault, DSBD_FAULT_NONFINITE);
      stamp(73);
      lmp = wave_max_f32(lmp); lmq = wave_max_f32(lmq);
      float* const wm = sh.wmax[(i - i_lo) & 1];       // two buffers: a wave is at most one row ahead of the slowest
      if (lane == 0) { wm[2 * wave] = lmp; wm[2 * wave + 1] = lmq; }
      __syncthreads();
#pragma unroll
      for (int w = 0; w < VL_WAVES; ++w) { lmp = fmaxf(lmp, wm[2 * w]); lmq = fmaxf(lmq, wm[2 * w + 1]); }
      const double mp = (double)lmp, mq = (double)lmq;
      if (tid == 0) { sh.lm_p[i - i_lo] = mp; sh.lm_q[i - i_lo] = mq; }
      // XU exponentials per model at a time (all of a round's at once would cost more registers than there are to spare)
#pragma unroll
      for (int k = 0; k < XU; ++k) {
        const int x = xA + k * VL_BLOCK;
        if (x < x_hi) {
          const double ep = exp_nonpos((double)fpA[k] - mp, sh.exp_tab);
          double eq = ep;
          if (!a.alias) eq = exp_nonpos((double)fqA[k] - mq, sh.exp_tab);
          store(joff + x, ep, eq);
          s_p += ep; s_q += eq;
        }
      }
      __builtin_amdgcn_sched_barrier(0);
      if (haveB) {
#pragma unroll
        for (int k = 0; k < XU; ++k) {
          const int x = xB + k * VL_BLOCK;
          if (x < x_hi) {
            const double ep = exp_nonpos((double)fpB[k] - mp, sh.exp_tab);
            double eq = ep;
            if (!a.alias) eq = exp_nonpos((double)fqB[k] - mq, sh.exp_tab);
            store(joff + x, ep, eq);
            s_p += ep; s_q += eq;
          }
        }
      }
      // the rest of a long piece, read a second time (from the caches): XU logits of each model at a time, the next
      // round's requested before this round's exponentials are taken; ragged end predicated
      {
        int x = xB + XU * VL_BLOCK;
        float np[XU], nq[XU];
        if (x < x_hi) {
#pragma unroll
          for (int k = 0; k < XU; ++k) {
            const int xx = min(x + k * VL_BLOCK, x_hi - 1);
            np[k] = zp[xx]; nq[k] = zq[xx];
          }
        }
        while (x < x_hi) {
          float fp[XU], fq[XU];
#pragma unroll
          for (int k = 0; k < XU; ++k) { fp[k] = np[k]; fq[k] = nq[k]; }
          const int xn = x + XU * VL_BLOCK;
          if (xn < x_hi) {
#pragma unroll
            for (int k = 0; k < XU; ++k) {
              const int xx = min(xn + k * VL_BLOCK, x_hi - 1);
              np[k] = zp[xx]; nq[k] = zq[xx];
            }
          }
#pragma unroll
          for (int k = 0; k < XU; ++k) {
            if (x + k * VL_BLOCK < x_hi) {
              const double ep = exp_nonpos((double)fp[k] - mp, sh.exp_tab);
              double eq = ep;
              if (!a.alias) eq = exp_nonpos((double)fq[k] - mq, sh.exp_tab);
              store(joff + x + k * VL_BLOCK, ep, eq);
              s_p += ep; s_q += eq;
            }
          }
          x = xn;
        }
      }
      };
      // (an aliased q_beam is p_beam: both stores then go to one place)
      if (in_lds) exp_pass([&](long long jj, double ep, double eq) { pl[(int)jj] = ep; ql[(int)jj] = eq; });
      else if (n_lds == 0) exp_pass([&](long long jj, double ep, double eq) { pbg[jj] = ep; qbg[jj] = eq; });
      else exp_pass([&](long long jj, double ep, double eq) {
        if (jj < n_lds) { pl[(int)jj] = ep; ql[(int)jj] = eq; } else { pbg[jj] = ep; qbg[jj] = eq; }
      });
      s_p = wave_sum(s_p);
      s_q = wave_sum(s_q);
      if (lane == 0) {
        sh.u.wpart[((i - i_lo) * VL_WAVES + wave) * 2] = s_p;
        sh.u.wpart[((i - i_lo) * VL_WAVES + wave) * 2 + 1] = s_q;
      }
    }
    stamp(100);
    __syncthreads();
    // ===== all-reduce of the rows' maxima and sums.  Only the workgroups that hold a piece of row i post its four
    // values (sum and maximum of the piece, both models) and only those are polled.
    epoch += 1;
    const unsigned long long rs_tag = exchange_tag(nonce + epoch);
    Slot* const rs_bank = slots + a.sl.r + (long long)(l - 1) * a.sl.r_stride;
    if (tid < 4 * (i_hi - i_lo + 1) && !(l == 1 && (int)blockIdx.x == a.mute_wg)) {
      const int r = tid >> 2, which = tid & 3;
      double v;
      if (which < 2) {
        const double* wp = &sh.u.wpart[r * VL_WAVES * 2 + which];
        v = ((wp[0] + wp[2]) + (wp[4] + wp[6])) + ((wp[8] + wp[10]) + (wp[12] + wp[14]));
      } else {
        v = which == 2 ? sh.lm_p[r] : sh.lm_q[r];
      }
      slot_post(rs_bank + (long long)g * a.sl.r_w + 4 * i_lo + tid, v, rs_tag);
    }
    stamp(102);

    if (l == 1 && g != 0 && wave == 2 && lane < 2 * NACC) {      // the accumulator words' values at launch
      double v = 0.0;
      if (!slot_wait(slots + a.sl.acc0 + lane, acc0_tag, v, a.sync_limit)) give_up();
      (&sh.acc_prev[0][0])[lane] = (unsigned long long)__double_as_longlong(v);
    }
    // ===== meanwhile: beam weights = softmax of the cumulative likelihoods over I (Section 2.1), by one wave
    if (wave == 1) {
      const bool valid = lane < nI;
      double mp = -INFINITY, mq = -INFINITY;
      for (int i = 0; i < nI; ++i) { mp = fmax(mp, sh.cum_p[i]); mq = fmax(mq, sh.cum_q[i]); }
      const double ep = valid ? exp_nonpos(sh.cum_p[lane] - mp, sh.exp_tab) : 0.0;
      const double eq = valid ? exp_nonpos(sh.cum_q[lane] - mq, sh.exp_tab) : 0.0;
      const double zp = wave_sum(ep), zq = wave_sum(eq);
      if (valid) { sh.bw_p[lane] = ep / zp; sh.bw_q[lane] = eq / zq; }
      // no beam of the layer with a likelihood above 0 under one of the models (stored likelihoods of -Inf), or a
      // likelihood that is no number: the joint is 0/0
      const bool lost = !(mp > -INFINITY && mp < INFINITY && mq > -INFINITY && mq < INFINITY) ||
                        __ballot(valid && (sh.cum_p[min(lane, 63)] != sh.cum_p[min(lane, 63)] ||
                                           sh.cum_q[min(lane, 63)] != sh.cum_q[min(lane, 63)])) != 0ull;
      if (lost && g == 0 && lane == 0) atomicOr(a.fault, DSBD_FAULT_NONFINITE);
    }

    // ===== and candidates = depth-l nodes whose parent is an input beam, in (rank, node) order
    int M = 0;
    float czp = 0.f, czq = 0.f;
    if (!bonus) {
      if (tid == 0) sh.counter = 0;
      __syncthreads();
      if (tid < n_pn && (sh.n_depth[tid] & NODE_DEPTH_MASK) == l) {
        const int n = n_begin + tid;
        const int par = sh.n_parent[tid];
        const bool cand = par >= n_begin && par < n && sh.slot_of[par - n_begin] >= 0;
        if (cand) sh.S_tmp[atomicAdd(&sh.counter, 1)] = n;
        else if (g == 0) a.out.node_status[n] = DSBD_PRUNED;
      }
      __syncthreads();
      M = sh.counter;
      if (tid < M) {
        const int n = sh.S_tmp[tid];
        const int rk = sh.n_rank[n - n_begin];
        int pos = 0;
        for (int j = 0; j < M; ++j) {
          const int n2 = sh.S_tmp[j];
          const int rk2 = sh.n_rank[n2 - n_begin];
          pos += (rk2 < rk) || (rk2 == rk && n2 < n);
        }
        sh.S_node[pos] = n;
      }
      __syncthreads();
      if (tid < M) {      // logits at the candidate's (parent beam, token): in flight while the row sums arrive
        const int n = sh.S_node[tid];
        const int par = sh.n_parent[n - n_begin];
        const int tok = sh.n_token[n - n_begin];
        czp = a.zp[(long long)par * V + tok];
        czq = a.zq[(long long)par * V + tok];
      }
    }

    // ===== rows' maxima and totals: thread (r, c) gathers column c = (row, model) from every R-th workgroup that holds
    // part of it and folds the pieces (sum relative to the piece's maximum) as it goes; the R partial results of a
    // column sit in R neighbouring lanes of one wave and are put on the column's maximum and added up by lane
    // exchanges that pair the lanes symmetrically (no table in the LDS, no barrier in between): every lane of a
    // column, in every workgroup of the prompt, gets the same bits.
    bool warp_pieces = false;               // warping: the table of the workgroups' largest entries is filled
    if constexpr (WARP) {
      if (tid < 256) { sh.gpart[tid] = -1.0; sh.ptot[tid] = -1.0; }     // (workgroups without a piece keep this)
      lds_barrier();                          // (the gathering threads below write other entries than their own)
    }
    {
      const int ncols = 2 * nI;
      int cshift = 0;
      while ((1 << cshift) < ncols) ++cshift;
      const int cpow = 1 << cshift;
      const int R = min(32, VL_BLOCK / cpow);                        // a power of two, 4 .. 32
      int rshift = 2;
      while ((1 << rshift) < R) ++rshift;
      const int r = tid & (R - 1), c = tid >> rshift;                // c < VL_BLOCK / R, which is at least cpow
      double accM = -INFINITY, accS = 0.0;
      bool mine = true;
      if (c < ncols) {
        const int i = c >> 1;
        const int w_lo = cut.rows_per_wg > 0 ? i / cut.rows_per_wg : i * cut.wg_per_row;
        const int w_hi = cut.rows_per_wg > 0 ? w_lo : w_lo + geo_pieces - 1;
        for (int w = w_lo + r; w <= w_hi; w += R) {
          double vs = 0.0, vm = 0.0;
          Slot* const sl0 = rs_bank + (long long)w * a.sl.r_w + 4 * i + (c & 1);
          mine = mine && slot_wait2(sl0, sl0 + 2, rs_tag, vs, vm, a.sync_limit);
          if constexpr (WARP) {              // (kept for the table of the workgroups' largest entries, below)
            if (cut.rows_per_wg == 0) ((c & 1) ? sh.ptot : sh.gpart)[min(w, 255)] = vm;
          }
          const double Mn = fmax(accM, vm);
          accS = accS * exp_nonpos(accM - Mn, sh.exp_tab) + vs * exp_nonpos(vm - Mn, sh.exp_tab);
          accM = Mn;
        }
      }
      stamp(20);
      if (!mine) give_up();
      // over aligned groups of R lanes: quads, the other quad of an eight, the other half of a sixteen (lane moves
      // inside the SIMD), then the other sixteen (one LDS exchange)
      double cm = accM;
      cm = fmax(cm, dpp_move_f64<0xB1, 0xf>(cm));                    // quad_perm [1,0,3,2]
      cm = fmax(cm, dpp_move_f64<0x4E, 0xf>(cm));                    // quad_perm [2,3,0,1]
      if (R >= 8) cm = fmax(cm, dpp_move_f64<0x141, 0xf>(cm));       // row_half_mirror
      if (R >= 16) cm = fmax(cm, dpp_move_f64<0x140, 0xf>(cm));      // row_mirror
      if (R >= 32) cm = fmax(cm, __shfl_xor(cm, 16));
      double tot = accS * exp_nonpos(accM - cm, sh.exp_tab);         // partial results without a piece: 0 x exp(-inf) = 0
      tot += dpp_move_f64<0xB1, 0xf>(tot);
      tot += dpp_move_f64<0x4E, 0xf>(tot);
      if (R >= 8) tot += dpp_move_f64<0x141, 0xf>(tot);
      if (R >= 16) tot += dpp_move_f64<0x140, 0xf>(tot);
      if (R >= 32) tot += __shfl_xor(tot, 16);
      __syncthreads();                       // the beam weights (another wave's) are there; so is a give-up
      if (sh.abort) return;
      stamp(21);
      // column totals; the scale factors of the rows, and what the fp64 log-sum-exp needs (taken later)
      if (c < ncols && r == 0) {
        const int i = c >> 1;
        if (c & 1) { sh.max_q[i] = cm; sh.sq[i] = sh.bw_q[i] / tot; sh.lse_q[i] = tot; }
        else { sh.max_p[i] = cm; sh.sp[i] = sh.bw_p[i] / tot; sh.lse_p[i] = tot; }
      }
      // every workgroup's share of p_beam follows from its piece's sum: sampling from p_beam (the additional layer,
      // the draws that fill a layer up) then needs no exchange of the workgroups' totals.  Only where a gathering
      // thread holds exactly one piece (its sum and maximum are still in its registers).
      // (entries of workgroups without a piece are never written: the reader knows which those are)
      const bool single_piece = !WARP && cut.rows_per_wg == 0 && geo_pieces <= R;
      if (tid == 0) sh.ptot_ok = single_piece ? 1 : 0;
      if constexpr (WARP) {
        // Every workgroup's largest entry of either joint follows from what the gathering threads hold (a piece's
        // largest exponential is 1 against the piece's own maximum): p_beam's largest entry in the piece of row i is
        // (beam weight / row sum) exp(piece maximum - row maximum).  Every workgroup evaluates this alike, bit for
        // bit, for every workgroup of the prompt (rows cut into pieces, a piece per workgroup; with whole rows per
        // workgroup the table is left alone and the selection below takes its tree form).
        // (worth it with many more workgroups than entries to keep: the K-th largest of a few largest entries is a
        // poor bound.  Measured: 16 workgroups per prompt, K = 10: 247 us against the tree form's 202 us; 64
        // workgroups, K = 32: 177 against 167 us; 64 and K = 10: 115 against 131 us; 256 and K = 10: 146 against 176 us.)
        warp_pieces = cut.rows_per_wg == 0 && nI * geo_pieces >= 4 * a.top_k;
        if (warp_pieces && c < ncols) {
          const int i = c >> 1;
          const double scale = ((c & 1) ? sh.bw_q[i] : sh.bw_p[i]) / tot;
          double* const tab = (c & 1) ? sh.ptot : sh.gpart;
          const int w_lo = i * cut.wg_per_row, w_hi = w_lo + geo_pieces - 1;
          for (int w = w_lo + r; w <= w_hi; w += R) {        // the pieces this thread gathered: their maxima are in the table
            const double vm = tab[min(w, 255)];
            tab[min(w, 255)] = vm > -INFINITY ? scale * exp_nonpos(vm - cm, sh.exp_tab) : -1.0;     // (an empty piece holds nothing)
          }
        }
      }
      if (single_piece && c < ncols && (c & 1) == 0 && r < geo_pieces) {
        const int i = c >> 1;
        sh.ptot[i * cut.wg_per_row + r] = (sh.bw_p[i] / tot) * (accS * exp_nonpos(accM - cm, sh.exp_tab));
      }
      __syncthreads();
    }
    stamp(24);
    // scaling, fused with this thread's part of F(1) = sum max(p_beam - q_beam, 0) (second entry of the chain)
    double f1 = 0.0;
    double tmax_p = -1.0, tmax_q = -1.0;     // warping: the largest scaled entries this thread has seen
    // (the one-level selection of the warped kernel needs no scaled slices: it scales the few entries it compares
    // on the fly and the slices are dead afterwards; only its fallback, the tree form, runs this pass after all)
    const bool defer_scaling = WARP && a.warp_fast && a.G > 1 && warp_pieces;
    auto scale_pass = [&]() {
    for (int i = i_lo; i <= i_hi; ++i) {
      const long long j_lo = max(e_lo, (long long)i * V) - e_lo;
      const long long j_hi = min(e_hi, (long long)(i + 1) * V) - e_lo;
      // (the slice holds exponentials against the piece's own maximum: put them on the row's)
      const double fp = sh.sp[i] * exp_nonpos(sh.lm_p[i - i_lo] - sh.max_p[i], sh.exp_tab);
      const double fq = sh.sq[i] * exp_nonpos(sh.lm_q[i - i_lo] - sh.max_q[i], sh.exp_tab);
      with_slices([&](auto P, auto Q, long long r0, long long r1) {
        const long long j_end = min(j_hi, r1);
        long long j = max(j_lo, r0) + tid;
        for (; j + 3 * VL_BLOCK < j_end; j += 4 * VL_BLOCK) {      // four elements of each array in flight
          double pv[4], qv[4];
#pragma unroll
          for (int k = 0; k < 4; ++k) { pv[k] = P[j + k * VL_BLOCK]; qv[k] = Q[j + k * VL_BLOCK]; }
#pragma unroll
          for (int k = 0; k < 4; ++k) {
            pv[k] *= fp; qv[k] *= fq;
            P[j + k * VL_BLOCK] = pv[k]; Q[j + k * VL_BLOCK] = qv[k];
            if constexpr (WARP) { tmax_p = fmax(tmax_p, pv[k]); tmax_q = fmax(tmax_q, qv[k]); }
            else f1 += fmax(pv[k] - qv[k], 0.0);
          }
        }
        for (; j < j_end; j += VL_BLOCK) {
          const double pv = P[j] * fp, qv = Q[j] * fq;
          P[j] = pv; Q[j] = qv;
          if constexpr (WARP) { tmax_p = fmax(tmax_p, pv); tmax_q = fmax(tmax_q, qv); }
          else f1 += fmax(pv - qv, 0.0);
        }
      });
    }
    };
    if (!defer_scaling) scale_pass();
    if constexpr (WARP) {
      // ===== warping T: top-k / top-p on the two joints (Section 2.1; Section 3.1 "Details": p_beam = T o p/P).
      // Every workgroup finds the K first entries of its slice.  The lists travel up a tree: the first workgroup
      // of every group of WARP_GROUP merges its group's lists, the prompt's first workgroup merges the groups'
      // lists, cuts the result by top-p, renormalises and posts the surviving entries (at most 2K), which every
      // workgroup then holds: the rest of the layer needs no further exchange.
      __syncthreads();                       // the scaled slices are complete
      const int K = a.top_k;
      typedef __attribute__((address_space(3))) int lds_i32;
      // scratch (all rewritten later in the layer): candidates in S_pb/S_qb (values) and S_zp/S_zq (indices),
      // lists in Pa (values: p then q) and Pb (indices); collected lists in the dynamic LDS (the slices are not
      // needed any more by then): values [model][source * K + rank], then the indices
      lds_f64* const cvp = (lds_f64*)sh.S_pb; lds_f64* const cvq = (lds_f64*)sh.S_qb;
      lds_i32* const cip = (lds_i32*)sh.S_zp; lds_i32* const ciq = (lds_i32*)sh.S_zq;
      lds_f64* const lv = (lds_f64*)sh.Pa; lds_i32* const li = (lds_i32*)sh.Pb;
      lds_f64* const gv = (lds_f64*)dyn_lds;
      lds_i32* const gi = (lds_i32*)(dyn_lds + 2 * WARP_CAND);
      // The K first of na candidates by counting for each those ahead of it, eight threads per candidate and 64
      // candidates per pass; ranks nobody takes keep what the caller put there.
      auto rank_cands = [&](lds_f64* va, lds_i32* ia, int na, lds_f64* ov, lds_i32* oi) {
        const int part = tid & 7;
        for (int t0 = 0; t0 < na; t0 += VL_BLOCK / 8) {
          const int t = t0 + (tid >> 3);
          const bool has = t < na;
          const double v = has ? va[t] : 0.0;
          const int ix = has ? ia[t] : 0;
          int rank = 0;
          if (has) {
            int c = part;
            for (; c + 24 < na; c += 32) {     // four candidates per round, their loads in flight together
              double o[4];
              int oi4[4];
#pragma unroll
              for (int k = 0; k < 4; ++k) { o[k] = va[c + 8 * k]; oi4[k] = ia[c + 8 * k]; }
#pragma unroll
              for (int k = 0; k < 4; ++k) rank += cand_before(o[k], oi4[k], v, ix) ? 1 : 0;
            }
            for (; c < na; c += 8) rank += cand_before(va[c], ia[c], v, ix) ? 1 : 0;
          }
          rank += __shfl_xor(rank, 1);
          rank += __shfl_xor(rank, 2);
          rank += __shfl_xor(rank, 4);
          if (has && part == 0 && rank < K) { ov[rank] = v; oi[rank] = ix; }
        }
      };
      // candidates (counts in W_cnt) -> lists; missing ranks are "none" (-1, INT_MAX), which sorts last
      auto rank_select = [&]() {
        if (tid < 2 * K) { lv[tid] = -1.0; li[tid] = INT_MAX; }
        __syncthreads();
        rank_cands(cvp, cip, min(sh.W_cnt[0], WARP_CAND), lv, li);
        rank_cands(cvq, ciq, min(sh.W_cnt[1], WARP_CAND), lv + K, li + K);
      };
      // everything at or above the bounds W_tau is a candidate (counts in W_cnt; the arrays hold the first WARP_CAND)
      bool scaled = !defer_scaling;          // the slices hold joint entries (else exponentials against the piece's maximum)
      auto collect_at_or_above = [&]() {
        // (a little below the bounds: the values compared here and the ones the candidates are ranked by, below, may
        // differ in the last bits)
        const double tp = sh.W_tau[0] * (1.0 - 1e-12), tq = sh.W_tau[1] * (1.0 - 1e-12);
        // (unscaled slices: one piece of one row per workgroup; the same products as the scaling pass forms)
        double mp = 1.0, mq = 1.0;
        if (!scaled && i_lo <= i_hi) {
          mp = sh.sp[i_lo] * exp_nonpos(sh.lm_p[0] - sh.max_p[i_lo], sh.exp_tab);
          mq = sh.sq[i_lo] * exp_nonpos(sh.lm_q[0] - sh.max_q[i_lo], sh.exp_tab);
        }
        auto offer = [&](long long j, double vp_raw, double vq_raw) {
          const double vp = vp_raw * mp, vq = vq_raw * mq;
          if (vp >= tp) {
            const int c = atomicAdd(&sh.W_cnt[0], 1);
            if (c < WARP_CAND) { cvp[c] = vp; cip[c] = (int)(e_lo + j); }
          }
          if (vq >= tq) {
            const int c = atomicAdd(&sh.W_cnt[1], 1);
            if (c < WARP_CAND) { cvq[c] = vq; ciq[c] = (int)(e_lo + j); }
          }
        };
        with_slices([&](auto P, auto Q, long long r0, long long r1) {
          long long j = r0 + tid;
          for (; j + 3 * VL_BLOCK < r1; j += 4 * VL_BLOCK) {
            double pv[4], qv[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) { pv[k] = P[j + k * VL_BLOCK]; qv[k] = Q[j + k * VL_BLOCK]; }
#pragma unroll
            for (int k = 0; k < 4; ++k) offer(j + k * VL_BLOCK, pv[k], qv[k]);
          }
          for (; j < r1; j += VL_BLOCK) offer(j, P[j], Q[j]);
        });
      };
      // ===== One-level selection (many more workgroups per prompt than entries to keep).  A lower bound of the joint's
      // K-th entry comes from the table of every workgroup's largest entry, which every workgroup holds without an
      // exchange (filled where the row sums are gathered); one pass collects what the slice holds at or above it (a
      // handful of entries per prompt); the workgroups that can hold candidates post them, everybody collects and
      // ranks them itself: one exchange, no tree, and every workgroup ends up with the lists, so the result needs no
      // broadcast either.  If the candidates do not fit (a workgroup's share of the slots, 64 posting workgroups,
      // WARP_CAND entries in all: many equal values, or the large entries crowded into a few slices), every workgroup
      // sees that in the same counts and the tree form below takes over.  The candidates' slots are a region per
      // layer, written once per launch: only the workgroups that post are waited for, so a workgroup without
      // candidates (and, in a later layer, without a piece of a row) may still be reading a layer's lines when the
      // others have moved on.
      bool fast = a.warp_fast && a.G > 1 && warp_pieces;      // uniform over the prompt's workgroups
      bool fast_done = false;
      lds_f64* const all_p = (lds_f64*)sh.gpart;        // [G] every workgroup's largest entry of p_beam ...
      lds_f64* const all_q = (lds_f64*)sh.ptot;         // ... and of q_beam (-1: the workgroup holds nothing)
      lds_f64* const stage = (lds_f64*)sh.tsum;         // [64][8] first lines of the workgroups that hold candidates
      lds_i32* const wl = (lds_i32*)sh.A_idx;           // [64] those workgroups
      lds_f64* const off_p = (lds_f64*)sh.A_cum_p;      // [64] where their candidates go in the joint lists ...
      lds_f64* const off_q = (lds_f64*)sh.A_cum_q;      // ... (as doubles: small integers, exact)
      const double slack = 1.0 - 1e-12;                 // (a workgroup's own largest entry may differ from the table's in the last bit)
      unsigned long long tag_w = 0;
      int nW = 0;
      while (true) {
        // ---- the bounds W_tau
        if (fast) {
          // The K-th largest of the workgroups' largest entries, or anything below it, is a lower bound of the joint's
          // K-th entry (K entries of K different workgroups are at or above it).  One wave per model finds it;
          // fewer than K values leave -1: everything passes, the counts below show it, and the tree form takes over.
          tag_w = exchange_tag(nonce + epoch + 1);
          epoch += 1;
          if (tid < 2) sh.W_cnt[tid] = 0;
          if (wave < 2) {
            lds_f64* const arr = wave ? all_q : all_p;
            // (as 32-bit patterns of the values rounded down to floats, which order like the values; the answer is
            // built from the leading bit down: the largest pattern, its low 12 bits zero, that K values reach)
            unsigned int key[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
              const int w = lane * 4 + k;
              const double v = w < a.G ? arr[w] : -1.0;
              key[k] = v > 0.0 ? (unsigned int)__float_as_int(__double2float_rd(v)) : 0u;
            }
            unsigned int prefix = 0;
#pragma unroll 1
            for (int b = 30; b >= 12; --b) {
              const unsigned int cand = prefix | (1u << b);
              const int cnt = __popcll(__ballot(key[0] >= cand)) + __popcll(__ballot(key[1] >= cand)) +
                              __popcll(__ballot(key[2] >= cand)) + __popcll(__ballot(key[3] >= cand));
              if (cnt >= K) prefix = cand;
            }
            const float kth = prefix ? __int_as_float((int)prefix) : -1.0f;    // fewer than K values: everything passes
            if (lane == 0) sh.W_tau[wave] = (double)kth;
          }
          __syncthreads();
          stamp(57);
          // the workgroups that can hold candidates (by the table, with a little slack), in workgroup order
          {
            const double tp = sh.W_tau[0] * slack, tq = sh.W_tau[1] * slack;
            const bool flagged = tid < a.G && (all_p[min(tid, 255)] >= tp || all_q[min(tid, 255)] >= tq);
            const unsigned long long fm = __ballot(flagged);
            if (lane == 0) sh.scan_w[wave] = (double)__popcll(fm);
            __syncthreads();
            int before = 0, all = 0;
#pragma unroll
            for (int w = 0; w < VL_WAVES; ++w) { const int cw = (int)sh.scan_w[w]; before += w < wave ? cw : 0; all += cw; }
            const int pos = before + __popcll(fm & ((1ull << lane) - 1ull));
            if (flagged && pos < 64) wl[pos] = tid;
            nW = all;
          }
        } else {
          // Tree form (1): a lower bound of the slice's K-th entry: the K-th largest of the maxima of 64 groups of
          // eight threads (K of the slice's entries, from different groups, are at or above it)
          double gp = tmax_p, gq = tmax_q;
#pragma unroll
          for (int off = 1; off <= 4; off <<= 1) { gp = fmax(gp, __shfl_xor(gp, off)); gq = fmax(gq, __shfl_xor(gq, off)); }
          if ((lane & 7) == 0) { sh.tsum[wave * 8 + (lane >> 3)] = gp; sh.tsum[64 + wave * 8 + (lane >> 3)] = gq; }
          if (tid < 2) sh.W_cnt[tid] = 0;
          __syncthreads();
          stamp(57);
          // four threads count, for one of the 2 x 64 maxima, those ahead of it; the one with K - 1 ahead is the bound
          const int m = tid >> 8, i = (tid >> 2) & 63, part = tid & 3;
          const double v = sh.tsum[m * 64 + i];
          int rank = 0;
#pragma unroll
          for (int j = 0; j < 16; ++j) {
            const int c = part + 4 * j;
            const double o = sh.tsum[m * 64 + c];
            rank += (o > v || (o == v && c < i)) ? 1 : 0;
          }
          rank += __shfl_xor(rank, 1);
          rank += __shfl_xor(rank, 2);
          if (part == 0 && rank == K - 1) sh.W_tau[m] = v;    // -1 when fewer than K groups hold anything: everything passes
        }
        __syncthreads();
        stamp(58);
        collect_at_or_above();               // (2) everything at or above the bound is a candidate
        __syncthreads();
        // The candidates are ranked by value, equal values by index, and equal logits of a row must give equal
        // values for that wherever in the row they sit (logits that came out of 16-bit arithmetic tie all the time).
        // A slice entry is exp(z - piece maximum) x a factor of the piece: two roundings that differ from piece to
        // piece.  So the few candidates get their value once more from the logit itself, in the one form that
        // depends on the row only (the form the candidates of the accept tests use as well).  (Taken inside the
        // pass above, by the thread that finds a candidate, it measured no faster, and slower with many candidates.)
        auto canonical_values = [&]() {
          const int n_p = min(sh.W_cnt[0], WARP_CAND), n_q = min(sh.W_cnt[1], WARP_CAND);
          for (int t = tid; t < n_p + n_q; t += VL_BLOCK) {
            const bool is_q = t >= n_p;
            const int c = is_q ? t - n_p : t;
            const int flat = is_q ? ciq[c] : cip[c];
            if (flat < 0 || (long long)flat >= (long long)nI * V) continue;       // ("none": nothing to look up)
            const int i = (int)div_floor(flat, V);
            const int x = flat - i * V;
            const float z = (is_q ? a.zq : a.zp)[(long long)sh.I_node[i] * V + x];
            const double v = exp_nonpos((double)z - (is_q ? sh.max_q[i] : sh.max_p[i]), sh.exp_tab) * (is_q ? sh.sq[i] : sh.sp[i]);
            if (is_q) cvq[c] = v; else cvp[c] = v;
          }
        };
        canonical_values();
        __syncthreads();
        stamp(60);
        if (fast) {
          // ---- the candidates of the workgroups that can hold any: counts and the first three in the first line
          // of the workgroup's slots (one round trip for nearly everything), the rest behind it
          const int cp = sh.W_cnt[0], cq = sh.W_cnt[1];
          const int room = (a.sl.b_w - 2) / 2;             // entries a workgroup can post
          const bool post = all_p[g] >= sh.W_tau[0] * slack || all_q[g] >= sh.W_tau[1] * slack;
          Slot* const wb_l = slots + a.sl.wb + (long long)(l - 1) * a.sl.wb_stride;     // this layer's region
          Slot* const mine = wb_l + (long long)g * a.sl.b_w;
          const int n_posted = cp + cq <= room ? cp + cq : 0;
          if (post && tid < max(8, 2 + 2 * n_posted)) {
            double payload;
            if (tid < 2) payload = (double)(tid ? cq : cp);
            else {
              const int e = (tid - 2) >> 1;
              if (e >= n_posted) payload = -1.0;
              else payload = (tid & 1) ? (double)(e < cp ? cip[e] : ciq[e - cp]) : (e < cp ? cvp[e] : cvq[e - cp]);
            }
            slot_post(mine + tid, payload, tag_w);
          }
          const int n_poll = 8 * min(nW, 64);
          for (int t = tid; t < n_poll; t += VL_BLOCK) {
            double v = 0.0;
            if (!slot_wait(wb_l + (long long)wl[t >> 3] * a.sl.b_w + (t & 7), tag_w, v, a.sync_limit)) give_up();
            stage[t] = v;
          }
          __syncthreads();                                 // (also: everybody has posted from the candidate arrays)
          if (sh.abort) return;
          stamp(62);
          if (wave < 2) {                                  // where every workgroup's candidates go, a wave per model
            const bool in = lane < min(nW, 64);
            const double mine_c = in ? stage[lane * 8 + wave] : 0.0;
            const bool crowded = in && stage[lane * 8] + stage[lane * 8 + 1] > (double)room;
            const double incl = wave_inclusive_scan(mine_c);
            if (in) (wave ? off_q : off_p)[lane] = incl - mine_c;
            const double total = __shfl(incl, 63);
            const bool bad_w = __ballot(crowded) != 0ull || total > (double)WARP_CAND || nW > 64;
            if (lane == 0) { sh.W_cnt[wave] = (int)total; sh.state[wave] = bad_w ? 1 : 0; }
          }
          __syncthreads();
          const bool crowded_any = (sh.state[0] | sh.state[1]) != 0;
          if (crowded_any) {                               // the same counts in every workgroup: all take the tree form
            __syncthreads();                               // (the flags are read; the tree form writes them again)
            if (!scaled) { scale_pass(); scaled = true; __syncthreads(); }
            fast = false;
            continue;
          }
          for (int t = tid; t < nW * 64; t += VL_BLOCK) {      // (room < 64)
            const int j = t >> 6, e = t & 63;
            const int cpj = (int)stage[j * 8], cqj = (int)stage[j * 8 + 1];
            if (e >= cpj + cqj) continue;
            double v, ix;
            if (e < 3) { v = stage[j * 8 + 2 + 2 * e]; ix = stage[j * 8 + 3 + 2 * e]; }
            else {
              Slot* const at = wb_l + (long long)wl[j] * a.sl.b_w + 2 + 2 * e;
              v = 0.0; ix = 0.0;
              if (!slot_wait2(at, at + 1, tag_w, v, ix, a.sync_limit)) give_up();
            }
            if (e < cpj) { const int at_l = (int)off_p[j] + e; cvp[at_l] = v; cip[at_l] = (int)ix; }
            else { const int at_l = (int)off_q[j] + e - cpj; cvq[at_l] = v; ciq[at_l] = (int)ix; }
          }
          __syncthreads();
          if (sh.abort) return;
          stamp(63);
        } else if (sh.W_cnt[0] > WARP_CAND || sh.W_cnt[1] > WARP_CAND) {
          // too many entries at or above the bound (many equal values, or a vocabulary of a few hundred tokens):
          // every wave extracts the K first of its lanes' elements a rank at a time; those become the candidates
          __syncthreads();                     // everybody has read the counts
          double pv_prev = INFINITY, qv_prev = INFINITY;
          int pi_prev = -1, qi_prev = -1;
          for (int r = 0; r < K; ++r) {
            double bp = -1.0, bq = -1.0;
            int ip = INT_MAX, iq = INT_MAX;
            for (long long j = tid; j < len; j += VL_BLOCK) {
              const int fi = (int)(e_lo + j);
              const double vp = ldp(j), vq = ldq(j);
              if (cand_before(pv_prev, pi_prev, vp, fi) && cand_before(vp, fi, bp, ip)) { bp = vp; ip = fi; }
              if (cand_before(qv_prev, qi_prev, vq, fi) && cand_before(vq, fi, bq, iq)) { bq = vq; iq = fi; }
            }
            wave_first(bp, ip);
            wave_first(bq, iq);
            if (lane == 0) { cvp[wave * K + r] = bp; cip[wave * K + r] = ip; cvq[wave * K + r] = bq; ciq[wave * K + r] = iq; }
            pv_prev = bp; pi_prev = ip; qv_prev = bq; qi_prev = iq;
          }
          if (tid < 2) sh.W_cnt[tid] = VL_WAVES * K;
          __syncthreads();
          canonical_values();
        }
        rank_select();                         // barrier inside, after the counts are final
        __syncthreads();
        stamp(61);
        fast_done = fast;
        break;
      }
      unsigned long long tag_d = 0;
      if (!fast_done) {
      // (3) up the tree.  A list travels as 4K words (model, rank, value | index).
      auto post_list = [&](Slot* where, unsigned long long tag) {
        if (tid < 4 * K) {
          const int m = tid / (2 * K), r = (tid % (2 * K)) >> 1;
          const double payload = (tid & 1) ? (double)li[m * K + r] : lv[m * K + r];
          slot_post(where + tid, payload, tag);
        }
      };
      // n_src lists, b_w slots apart from `from` on, into gv / gi; up to four slots in flight per thread
      auto collect_lists = [&](Slot* from, unsigned long long tag, int n_src) {
        const int nS = n_src * 4 * K;
        bool okc = true;
        for (int s0 = tid; s0 < nS && okc; s0 += 4 * VL_BLOCK) {
          bool have[4];
          double val[4];
#pragma unroll
          for (int k = 0; k < 4; ++k) { have[k] = s0 + k * VL_BLOCK >= nS; val[k] = 0.0; }
          long long t0 = 0;
          for (int spin = 0;; ++spin) {
            unsigned long long w0[4], w1[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
              w0[k] = 0; w1[k] = 0;
              if (!have[k]) {
                const int sk = s0 + k * VL_BLOCK;
                Slot* sl = from + (long long)(sk / (4 * K)) * a.sl.b_w + sk % (4 * K);
                w0[k] = __hip_atomic_load(&sl->w0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                w1[k] = __hip_atomic_load(&sl->w1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
              }
            }
#pragma unroll
            for (int k = 0; k < 4; ++k)
              if (!have[k] && (w0[k] ^ w1[k]) == tag) { val[k] = __longlong_as_double((long long)w0[k]); have[k] = true; }
            if (have[0] && have[1] && have[2] && have[3]) break;
            if (spin == 0) t0 = wall_clock64();
            else if ((spin & 15) == 0 && wall_clock64() - t0 > a.sync_limit) { okc = false; break; }
            __builtin_amdgcn_s_sleep(1);
          }
#pragma unroll
          for (int k = 0; k < 4; ++k) {
            const int sk = s0 + k * VL_BLOCK;
            if (sk < nS && okc) {
              const int src = sk / (4 * K), c = sk % (4 * K);
              const int m = c / (2 * K), r = (c % (2 * K)) >> 1;
              if (c & 1) gi[m * WARP_CAND + src * K + r] = (int)val[k];
              else gv[m * WARP_CAND + src * K + r] = val[k];
            }
          }
        }
        if (!okc) give_up();
      };
      // The K first of n_src <= 16 collected lists, each in rank order: one or two levels of four-way merges.  In
      // a merge an entry's rank is its own rank plus the numbers of entries of the three partner lists ahead of
      // it (binary searches, side by side, branch-free); ranks K and beyond drop out.
      auto merge_pass = [&](lds_f64* sv0, lds_i32* si0, lds_f64* sv1, lds_i32* si1, int n,
                            lds_f64* dv0, lds_i32* di0, lds_f64* dv1, lds_i32* di1) {
        for (int t = tid; t < 2 * n * K; t += VL_BLOCK) {
          const int m = t >= n * K ? 1 : 0, e = t - m * n * K;
          const int src = e / K, r = e - src * K;
          lds_f64* const sv = m ? sv1 : sv0;
          lds_i32* const si = m ? si1 : si0;
          const double v = sv[e];
          const int ix = si[e];
          // entries of a partner list ahead of this one: the longest leading part of which all are (steps 32,
          // 16, .. 1; a partner that does not exist has length 0 and is read at this entry's own list)
          int po[3], len_j[3], cnt[3];
#pragma unroll
          for (int j = 0; j < 3; ++j) {
            const int o = (src & ~3) + ((src + 1 + j) & 3);
            po[j] = (o < n ? o : src) * K; len_j[j] = o < n ? K : 0; cnt[j] = 0;
          }
#pragma unroll
          for (int step = 32; step >= 1; step >>= 1) {
            if (step > K) continue;          // uniform: short lists need fewer halvings
            double pv3[3];
            int pi3[3];
#pragma unroll
            for (int j = 0; j < 3; ++j) {
              const int at = min(cnt[j] + step - 1, K - 1);
              pv3[j] = sv[po[j] + at]; pi3[j] = si[po[j] + at];
            }
#pragma unroll
            for (int j = 0; j < 3; ++j)
              cnt[j] += ((cnt[j] + step - 1 < len_j[j]) & cand_before(pv3[j], pi3[j], v, ix)) ? step : 0;
          }
          const int rank = r + cnt[0] + cnt[1] + cnt[2];
          if (rank < K && ix != INT_MAX) {
            (m ? dv1 : dv0)[(src >> 2) * K + rank] = v;
            (m ? di1 : di0)[(src >> 2) * K + rank] = ix;
          }
        }
      };
      auto fill_none = [&](lds_f64* v0, lds_i32* i0, lds_f64* v1, lds_i32* i1, int cnt) {
        for (int t = tid; t < 2 * cnt; t += VL_BLOCK) {
          const int m = t >= cnt ? 1 : 0, e = t - m * cnt;
          (m ? v1 : v0)[e] = -1.0;
          (m ? i1 : i0)[e] = INT_MAX;
        }
      };
      // gv / gi -> lv / li.  The candidate arrays (first 4K entries per model) must hold "none" on entry: the
      // caller fills them before it collects, so that the barrier after the collection covers both.
      auto merge_lists = [&](int n) {
        if (n <= 4) {
          fill_none(lv, li, lv + K, li + K, K);
          __syncthreads();
          merge_pass(gv, gi, gv + WARP_CAND, gi + WARP_CAND, n, lv, li, lv + K, li + K);
          __syncthreads();
          return;
        }
        merge_pass(gv, gi, gv + WARP_CAND, gi + WARP_CAND, n, cvp, cip, cvq, ciq);
        fill_none(lv, li, lv + K, li + K, K);
        __syncthreads();
        merge_pass(cvp, cip, cvq, ciq, (n + 3) >> 2, lv, li, lv + K, li + K);
        __syncthreads();
      };
      if (a.G > 1) {
        const int first = g - g % WARP_GROUP;
        const int n_mem = min(WARP_GROUP, a.G - first);
        const int n_groups = (a.G + WARP_GROUP - 1) / WARP_GROUP;
        const unsigned long long tag_b = exchange_tag(nonce + epoch + 1), tag_c = exchange_tag(nonce + epoch + 2);
        tag_d = exchange_tag(nonce + epoch + 3);
        epoch += 3;
        post_list(slots + a.sl.b + (long long)g * a.sl.b_w, tag_b);
        if (g == first) {                    // the group's first workgroup merges the group's lists
          fill_none(cvp, cip, cvq, ciq, 4 * K);
          collect_lists(slots + a.sl.b + (long long)first * a.sl.b_w, tag_b, n_mem);
          __syncthreads();
          stamp(62);
          if (sh.abort) return;
          merge_lists(n_mem);
          stamp(63);
          if (n_groups > 1) post_list(slots + a.sl.c + (long long)(g / WARP_GROUP) * a.sl.b_w, tag_c);
        }
        if (g == 0 && n_groups > 1) {        // the prompt's first workgroup merges the groups' lists
          fill_none(cvp, cip, cvq, ciq, 4 * K);
          collect_lists(slots + a.sl.c, tag_c, n_groups);
          __syncthreads();
          stamp(64);
          if (sh.abort) return;
          merge_lists(n_groups);
        }
      }
      }   // (tree form)
      stamp(65);
      if (g == 0 || fast_done) {
        if (wave == 0) {
          // (4) top-p on the kept entries (rank order: the shortest leading part whose share exceeds top_p) and
          // renormalisation; lanes 0..31 carry p_beam's list, lanes 32..63 q_beam's, one rank each.  The running
          // sums add the entries one by one in rank order.
          const int r = lane & 31, half = lane & 32;
          const bool is_q = half != 0;
          const int ix = r < K ? li[(is_q ? K : 0) + r] : INT_MAX;
          const bool real = ix != INT_MAX;
          const double v = real ? lv[(is_q ? K : 0) + r] : 0.0;
          double cum = 0.0;
          int partner = -1;                  // lane of the other list's entry with the same index
          {
            // (the lists are read from the LDS, every lane of a half the same word: one read serves 32 lanes; lane
            // reads of the other lanes' registers cost a scalar round trip each)
            const int own = is_q ? K : 0, oth = is_q ? 0 : K;
            for (int c = 0; c < K; ++c) {
              const int i_own = li[own + c], i_oth = li[oth + c];
              const double v_own = i_own != INT_MAX ? lv[own + c] : 0.0;
              if (c <= r) cum += v_own;
              if (i_oth == ix) partner = (is_q ? 0 : 32) + c;
            }
          }
          const unsigned long long real_m = __ballot(real);
          const int n = __popcll(is_q ? (real_m >> 32) : (real_m & 0xffffffffull));     // real entries lead the list
          int keep = n;
          if (a.top_p < 1.0f) {
            const double mass = __shfl(cum, half + max(n - 1, 0));
            const unsigned long long over_m = __ballot(real && cum / mass > (double)a.top_p);
            const unsigned int mine = (unsigned int)(is_q ? (over_m >> 32) : (over_m & 0xffffffffull));
            if (mine) keep = __ffs((int)mine);
          }
          const double z = __shfl(cum, half + max(keep - 1, 0));
          const bool kept = r < keep;
          const double w = kept ? v / z : 0.0;
          // (5) union of the two supports, ascending flat index: a q entry whose index p_beam also keeps is
          // carried by the p entry
          const double w_partner = __shfl(w, max(partner, 0));       // 0 when the partner was cut
          const int kept_partner = __shfl((int)kept, max(partner, 0));
          const bool both = real && partner >= 0 && kept_partner;
          const double other = (both && !is_q) ? w_partner : 0.0;
          const bool valid = kept && !(is_q && both);
          int rank = 0;
          {
            // the valid entries' indices side by side in the LDS (lane c: p_beam's list, 32 + c: q_beam's)
            lds_i32* const vx = (lds_i32*)sh.A_idx;
            vx[lane] = valid ? ix : INT_MAX;
            wave_lds_fence();
            for (int c = 0; c < K; ++c) rank += (vx[c] < ix ? 1 : 0) + (vx[32 + c] < ix ? 1 : 0);
          }
          if (valid) { sh.U_idx[rank] = ix; sh.U_p[rank] = is_q ? 0.0 : w; sh.U_q[rank] = is_q ? w : other; }
          const unsigned long long vm = __ballot(valid);
          if (lane == 0) sh.nU = __popcll(vm);
        }
        __syncthreads();
        if (!fast_done && a.G > 1 && tid < 1 + 6 * K) {          // (6) ... and down again: the count, then (index, p, q) of at most 2K entries
          const int u = (tid - 1) / 3, f = (tid - 1) % 3;
          double payload = 0.0;
          if (tid == 0) payload = (double)sh.nU;
          else if (u < sh.nU) payload = f == 0 ? (double)sh.U_idx[u] : (f == 1 ? sh.U_p[u] : sh.U_q[u]);
          slot_post(slots + a.sl.d + tid, payload, tag_d);
        }
      } else {
        if (tid < 1 + 6 * K) {
          double v = 0.0;
          if (!slot_wait(slots + a.sl.d + tid, tag_d, v, a.sync_limit)) give_up();
          const int u = (tid - 1) / 3, f = (tid - 1) % 3;
          if (tid == 0) sh.nU = (int)v;
          else if (f == 0) sh.U_idx[u] = (int)v;
          else if (f == 1) sh.U_p[u] = v;
          else sh.U_q[u] = v;
        }
        __syncthreads();
        if (sh.abort) return;
      }
    }
    stamp(25);
    // p_beam and q_beam at every candidate's (parent beam, token)
    if (tid < M) {
      const int n = sh.S_node[tid];
      const int slot = sh.slot_of[sh.n_parent[n - n_begin] - n_begin];
      sh.S_zp[tid] = czp; sh.S_zq[tid] = czq;
      double pbx, qbx;
      if constexpr (WARP) {       // warped joints: the surviving entries, zero elsewhere
        const int flat = slot * V + sh.n_token[n - n_begin];
        int at = 0;                                  // entries with a smaller index (the list is in index order)
#pragma unroll
        for (int step = 32; step >= 1; step >>= 1) {
          const int probe = at + step - 1;
          at += (probe < sh.nU && sh.U_idx[min(probe, 63)] < flat) ? step : 0;
        }
        const bool hit = at < sh.nU && sh.U_idx[min(at, 63)] == flat;
        pbx = hit ? sh.U_p[min(at, 63)] : 0.0;
        qbx = hit ? sh.U_q[min(at, 63)] : 0.0;
      } else {
        pbx = exp_nonpos((double)czp - sh.max_p[slot], sh.exp_tab) * sh.sp[slot];
        qbx = exp_nonpos((double)czq - sh.max_q[slot], sh.exp_tab) * sh.sq[slot];
      }
      const float uf = sh.n_u[n - n_begin];
      // the test with p' = p_beam (first candidate, and every candidate right after an acceptance) needs no chain
      const double ratio = (qbx == 0.0) ? INFINITY : pbx / qbx;
      sh.S_pb[tid] = pbx; sh.S_qb[tid] = qbx; sh.S_u[tid] = uf;
      sh.S_flag[tid] = (unsigned char)(((double)uf <= ratio ? 1 : 0) | (fabs(ratio - (double)uf) <= NEAR_TIE ? 2 : 0));
    }
    if (tid == 0) { sh.cc[1] = 0.0; sh.FF[1] = 1.0; sh.kmax = 1; sh.acc_n = 0; sh.pos = 0; sh.kidx = 1; }
    // Entry 2 of the residual chain (c = 1) is needed by the first rejection of nearly every layer: its partial
    // sums are posted ahead of time and collected only when it is asked for.
    bool spec = false;
    Slot* spec_bank = nullptr;
    Slot* spec_gbank = nullptr;
    unsigned long long spec_tag = 0;
    double spec_own = 0.0;
    stamp(26);
    if (!WARP && M > 0) {
      const double tot = wg_total(f1);      // barrier inside: also publishes the scaled slices
      stamp(27);
      epoch += 1;
      spec_tag = exchange_tag(nonce + epoch);
      spec_bank = slots + a.sl.s + (long long)(l - 1) * a.sl.s_stride;
      spec_gbank = slots + a.sl.sc + (long long)(l - 1) * a.sl.sc_stride;
      if (tid == 0) dense_post(spec_bank, a.G, g, tot, spec_tag);
      spec_own = tot;
      spec = true;
    } else {
      __syncthreads();
    }

    // fp64 log-sum-exp of the input beams' rows: needed at the end of the layer only, so one wave takes the
    // logarithms while the first wave is busy with the decisions (or the others with the sampling prefix sums)
    if (wave == 1 && lane < nI) {
      sh.lse_p[lane] = sh.max_p[lane] + log(sh.lse_p[lane]);
      sh.lse_q[lane] = sh.max_q[lane] + log(sh.lse_q[lane]);
    }
    stamp(22);
    // sum over the slice of max(p_beam - c q_beam, 0); four loads in flight per thread
    // (the threads t0 .. t0+nt-1 share the work; the others return 0)
    auto slice_sum = [&](double c, int t0, int nt) -> double {
      double s0 = 0.0, s1 = 0.0, s2 = 0.0, s3 = 0.0;
      if (tid < t0) return 0.0;
      if constexpr (WARP) {       // the whole (warped) joint is the short list every workgroup holds
        const int c2 = tid - t0;
        return c2 < sh.nU ? fmax(sh.U_p[c2] - c * sh.U_q[c2], 0.0) : 0.0;
      }
      with_slices([&](auto P, auto Q, long long r0, long long r1) {
        // four elements of each array in flight per thread, the ragged end predicated (one element after the other,
        // the tail of a 4008-entry slice cost four dependent LDS round trips per chain entry; eight in flight cost
        // more registers than the kernel can spare beside the statistics pass)
        const int n = (int)r1;             // a slice has fewer than 2^31 entries
        const int j_first = (int)r0 + tid - t0;
        if constexpr (std::is_same<decltype(P), glb_f64*>::value) {
          // the part in the workspace (read through the caches): eight of each array in flight
          for (int j = j_first; j < n; j += 8 * nt) {
            double pv[8], qv[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) { const int jk = min(j + k * nt, n - 1); pv[k] = P[jk]; qv[k] = Q[jk]; }
#pragma unroll
            for (int k = 0; k < 8; k += 4) {
              s0 += (j + k * nt < n) ? fmax(pv[k] - c * qv[k], 0.0) : 0.0;
              s1 += (j + (k + 1) * nt < n) ? fmax(pv[k + 1] - c * qv[k + 1], 0.0) : 0.0;
              s2 += (j + (k + 2) * nt < n) ? fmax(pv[k + 2] - c * qv[k + 2], 0.0) : 0.0;
              s3 += (j + (k + 3) * nt < n) ? fmax(pv[k + 3] - c * qv[k + 3], 0.0) : 0.0;
            }
          }
        } else {
          for (int j = j_first; j < n; j += 4 * nt) {
            const int j1 = min(j + nt, n - 1), j2 = min(j + 2 * nt, n - 1), j3 = min(j + 3 * nt, n - 1);
            const double p0 = P[j], p1 = P[j1], p2 = P[j2], p3 = P[j3];
            const double q0 = Q[j], q1 = Q[j1], q2 = Q[j2], q3 = Q[j3];
            s0 += fmax(p0 - c * q0, 0.0);
            s1 += (j + nt < n) ? fmax(p1 - c * q1, 0.0) : 0.0;
            s2 += (j + 2 * nt < n) ? fmax(p2 - c * q2, 0.0) : 0.0;
            s3 += (j + 3 * nt < n) ? fmax(p3 - c * q3, 0.0) : 0.0;
          }
        }
      });
      return (s0 + s1) + (s2 + s3);
    };

    // Draws `cnt` samples (uniforms u[0..cnt)) from the weights max(p_beam - c q_beam, 0) (use_q) or p_beam over
    // I x V by inverse CDF in flat order; the workgroup owning a sample writes output slot out_base + j.
    auto draw = [&](double c, bool use_q, const float* u, int cnt, int out_base) -> bool {
      if constexpr (WARP) {
        // the weights live on the short list (ascending flat index) that every workgroup holds: one wave scans
        // it, the first workgroup writes the samples
        __syncthreads();           // the rows' log-sum-exps (another wave's work since the fold) are in place
        if (wave == 0) {
          const int nU = sh.nU;
          double w = 0.0;
          if (lane < nU) w = use_q ? fmax(sh.U_p[lane] - c * sh.U_q[lane], 0.0) : sh.U_p[lane];
          double incl = w;
          incl = wave_inclusive_scan(incl);
          const double Z = __shfl(incl, 63);
          const unsigned long long mass = __ballot(w > 0.0);
          for (int j = 0; j < cnt; ++j) {
            const double target = (double)u[j] * Z;
            const unsigned long long above = __ballot(incl > target);
            // the first entry whose inclusive prefix exceeds the target (rounding: the last one with mass)
            const int pl_ = above ? (int)__ffsll((long long)above) - 1 : (mass ? 63 - __clzll((long long)mass) : 0);
            if (g == 0 && lane == pl_) {
              const long long pick = sh.U_idx[pl_];
              const int i = (int)div_floor(pick, V);
              const int x = (int)(pick - (long long)i * V);
              const int node = sh.I_node[i];
              const long long o = (long long)prompt * a.W_cap + out_base + j;
              a.out.out_parent[o] = node;
              a.out.out_token[o] = x;
              a.out.out_node[o] = -1;
              const double lp_o = sh.cum_p[i] + ((double)a.zp[(long long)node * V + x] - sh.lse_p[i]);
              const double lq_o = sh.cum_q[i] + ((double)a.zq[(long long)node * V + x] - sh.lse_q[i]);
              a.out.out_logp_target[o] = lp_o;
              a.out.out_logp_draft[o] = lq_o;
              emit_next(out_base + j, node, x, lp_o, lq_o);
            }
          }
        }
        __syncthreads();
        return true;
      }
      float uj = 0.f;
      if (tid < cnt) uj = u[tid];
      // inclusive prefixes over this workgroup's threads (contiguous chunks) ...
      long long per = (len + VL_BLOCK - 1) / VL_BLOCK;
      if (!in_lds) {                      // slices in the workspace: chunks of a power of two (at least one) entries
        long long p2 = 1;
        while (p2 < per) p2 <<= 1;
        per = p2;
      }
      const long long t_lo = min(len, per * tid), t_hi = min(len, t_lo + per);   // slice-local
      double ts = 0.0;
      if (in_lds) {
        if (use_q) for (int j = (int)t_lo; j < (int)t_hi; ++j) ts += fmax((double)pl[j] - c * (double)ql[j], 0.0);
        else for (int j = (int)t_lo; j < (int)t_hi; ++j) ts += (double)pl[j];
      } else {
        // A thread walking its own chunk would make every load of a wave touch 64 cache lines (measured: 14 us for a
        // 16000-entry slice).  Instead a wave reads the 64 chunks of its threads 64 consecutive entries at a time and
        // adds them up across the lanes: `per` rounds, each holding 64 / per whole chunks or a 64th of one.
        const long long w_lo = per * 64 * wave;
        auto weight = [&](long long jj) -> double {
          if (jj >= len) return 0.0;
          if (jj < n_lds) return use_q ? fmax((double)pl[(int)jj] - c * (double)ql[(int)jj], 0.0) : (double)pl[(int)jj];
          return use_q ? fmax((double)pbg[jj] - c * (double)qbg[jj], 0.0) : (double)pbg[jj];
        };
        // eight rounds from r0 on (rounds beyond `lim` count nothing): one home for all eight in all but one group of
        // a wave, and then loads without branches between them, which the compiler keeps in flight together
        auto weights8 = [&](long long r0, long long lim, double (&w)[8]) {
          const long long b0 = w_lo + r0 * 64, b1 = w_lo + min(r0 + 8, lim) * 64;     // the group's range (uniform)
          if (b0 >= n_lds && b0 < len) {
#pragma unroll
            for (int k = 0; k < 8; ++k) {
              const long long jj = b0 + k * 64 + lane, jc = min(jj, len - 1);
              const double pv = pbg[jc], qv = use_q ? (double)qbg[jc] : 0.0;
              const double v = use_q ? fmax(pv - c * qv, 0.0) : pv;
              w[k] = (r0 + k < lim && jj < len) ? v : 0.0;
            }
          } else if (b1 <= n_lds) {
#pragma unroll
            for (int k = 0; k < 8; ++k) {
              const int jc = (int)min(b0 + k * 64 + lane, n_lds - 1);
              const double pv = pl[jc], qv = use_q ? (double)ql[jc] : 0.0;
              const double v = use_q ? fmax(pv - c * qv, 0.0) : pv;
              w[k] = (r0 + k < lim) ? v : 0.0;
            }
          } else {
#pragma unroll
            for (int k = 0; k < 8; ++k) w[k] = r0 + k < lim ? weight(b0 + k * 64 + lane) : 0.0;
          }
        };
        if (per < 64) {
          // sums over aligned groups of `per` lanes by lane moves inside the SIMD (one LDS exchange for groups of 32);
          // a group's first lane leaves the chunk's total in the table, where its thread picks it up
          const int S = 64 / (int)per;                  // chunks per round
          for (long long r0 = 0; r0 < per; r0 += 8) {
            double w[8];
            weights8(r0, per, w);
#pragma unroll
            for (int k = 0; k < 8; ++k) {
              double v = w[k];
              if (per >= 2) v += dpp_move_f64<0xB1, 0xf>(v);      // quad_perm [1,0,3,2]
              if (per >= 4) v += dpp_move_f64<0x4E, 0xf>(v);      // quad_perm [2,3,0,1]
              if (per >= 8) v += dpp_move_f64<0x141, 0xf>(v);     // row_half_mirror: the other quad of the eight
              if (per >= 16) v += dpp_move_f64<0x140, 0xf>(v);    // row_mirror: the other half of the sixteen
              if (per >= 32) v += __shfl_xor(v, 16);
              if (r0 + k < per && (lane & ((int)per - 1)) == 0)
                sh.tsum[wave * 64 + (int)(r0 + k) * S + lane / (int)per] = v;
            }
          }
          wave_lds_fence();
          ts = sh.tsum[tid];
        } else {
          const long long rpc = per / 64;                // rounds per chunk (a power of two); chunk after chunk
          double acc = 0.0;
          for (long long r0 = 0; r0 < per; r0 += 8) {
            double w[8];
            weights8(r0, per, w);                                                       // per >= 64 is a multiple of 8
#pragma unroll
            for (int k = 0; k < 8; ++k) {
              acc += w[k];
              if (((r0 + k + 1) & (rpc - 1)) == 0) {
                const double tot = wave_sum(acc);
                if (lane == (int)((r0 + k) / rpc)) ts = tot;
                acc = 0.0;
              }
            }
          }
        }
      }
      stamp(70);
      const double tincl = block_inclusive_scan(ts, sh);
      sh.tsum[tid] = tincl;
      if (tid == 0) sh.counter = 0;
      __syncthreads();
      // ... and over the workgroups (same order everywhere), gathered and scanned by one wave
      // (p_beam itself: the totals are known from the row sums, see above; the same in every workgroup of the prompt)
      const bool known_totals = !use_q && sh.ptot_ok != 0;
      unsigned long long tag = 0;
      Slot* bank = nullptr;
      if (!known_totals) {
        epoch += 1;
        tag = exchange_tag(nonce + epoch);
        bank = slots + bank_x(xchg++);
      }
      if (wave == 0) {
        double v[4];
        if (!known_totals) {
          const double mine = sh.tsum[VL_BLOCK - 1];
          if (lane == 0) dense_post(bank, a.G, g, mine, tag);
          if (!wave_collect4(bank, a.G, g, mine, tag, v, a.sync_limit)) give_up();
#pragma unroll
          for (int k = 0; k < 4; ++k) if (lane + 64 * k < a.G) sh.gpart[lane + 64 * k] = v[k];
          wave_lds_fence();          // now four consecutive workgroups per lane
        }
        lds_f64* const totals = known_totals ? (lds_f64*)sh.ptot : (lds_f64*)sh.gpart;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          const int w = 4 * lane + k;
          bool holds = w < a.G;
          if (known_totals) holds = holds && w / cut.wg_per_row < nI && w % cut.wg_per_row < geo_pieces;
          v[k] = holds ? (double)totals[w] : 0.0;
        }
        int nz = -1;                 // the last workgroup that holds any mass (uniform: from ballots)
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          const unsigned long long has = __ballot(v[k] > 0.0);
          if (has) nz = max(nz, 4 * (63 - __clzll((long long)has)) + k);
        }
        v[1] += v[0]; v[2] += v[1]; v[3] += v[2];
        double incl = v[3];
        incl = wave_inclusive_scan(incl);
        double excl = __shfl_up(incl, 1);
        if (lane == 0) excl = 0.0;
#pragma unroll
        for (int k = 0; k < 4; ++k) if (4 * lane + k < a.G) sh.gpart[4 * lane + k] = excl + v[k];
        if (lane == 0) sh.found = nz;
      }
      __syncthreads();
      stamp(71);
      if (sh.abort) return false;
      const double Z = sh.gpart[a.G - 1];
      const double before = g > 0 ? sh.gpart[g - 1] : 0.0;
      if (tid < cnt) {
        const double target = (double)uj * Z;
        sh.d_target[tid] = target;
        // owner: the first workgroup whose inclusive prefix exceeds the target (rounding: the last one with mass)
        int lo = 0, hi = a.G;
        while (lo < hi) { const int mid = (lo + hi) >> 1; if (sh.gpart[mid] > target) hi = mid; else lo = mid + 1; }
        const int owner = lo < a.G ? lo : max(sh.found, 0);
        if (owner == g) sh.S_tmp[atomicAdd(&sh.counter, 1)] = tid;
      }
      __syncthreads();
      stamp(72);
      const int n_mine = sh.counter;
      for (int k = 0; k < n_mine; ++k) {
        const int j = sh.S_tmp[k];
        const double target = sh.d_target[j];
        // the thread whose inclusive prefix is the first to exceed the target (rounding: the last one with mass,
        // found by the last thread)
        const bool above = before + sh.tsum[tid] > target;
        const bool prev_above = tid > 0 && (before + sh.tsum[tid - 1] > target);
        const bool holder = (above && !prev_above) || (tid == VL_BLOCK - 1 && !above);
        auto emit = [&](long long pick) {
          pick = min(pick + e_lo, total - 1);   // back to the flat index over I x V
          const int i = (int)div_floor(pick, V);
          const int x = (int)(pick - (long long)i * V);
          const int node = sh.I_node[i];
          const long long o = (long long)prompt * a.W_cap + out_base + j;
          a.out.out_parent[o] = node;
          a.out.out_token[o] = x;
          a.out.out_node[o] = -1;
          const double lp_o = sh.cum_p[i] + ((double)a.zp[(long long)node * V + x] - sh.lse_p[i]);
          const double lq_o = sh.cum_q[i] + ((double)a.zq[(long long)node * V + x] - sh.lse_q[i]);
          a.out.out_logp_target[o] = lp_o;
          a.out.out_logp_draft[o] = lq_o;
          emit_next(out_base + j, node, x, lp_o, lq_o);
        };
        if (in_lds) {
          if (holder) {
            int th = tid;
            if (!above)
              while (th > 0 && !(sh.tsum[th] > sh.tsum[th - 1])) --th;
            const long long c_lo = min(len, per * th), c_hi = min(len, c_lo + per);
            double accl = before + (th > 0 ? sh.tsum[th - 1] : 0.0);
            long long pick = -1, last = -1;
            for (long long jj = c_lo; jj < c_hi; ++jj) {
              const double v = use_q ? fmax((double)pl[(int)jj] - c * (double)ql[(int)jj], 0.0) : (double)pl[(int)jj];
              if (v > 0.0) last = jj;
              accl += v;
              if (accl > target) { pick = jj; break; }
            }
            if (pick < 0) pick = last >= 0 ? last : c_lo;
            emit(pick);
          }
        } else {
          // slices in the workspace: one thread walking its chunk would wait for a load per element, so the first wave
          // takes the chunk 64 entries at a time (coalesced loads, a scan across the lanes)
          if (holder) {
            int th = tid;
            if (!above)
              while (th > 0 && !(sh.tsum[th] > sh.tsum[th - 1])) --th;
            sh.pick_th = th;
          }
          __syncthreads();
          if (wave == 0) {
            const int th = sh.pick_th;
            const long long c_lo = min(len, per * th), c_hi = min(len, c_lo + per);
            double start = before + (th > 0 ? sh.tsum[th - 1] : 0.0);
            long long pick = -1, last = -1;
            for (long long b0 = c_lo; b0 < c_hi && pick < 0; b0 += 64) {
              const long long jj = b0 + lane;
              double v = 0.0;
              if (jj < c_hi) v = use_q ? fmax(ldp(jj) - c * ldq(jj), 0.0) : ldp(jj);
              double incl = v;
              incl = wave_inclusive_scan(incl);
              const unsigned long long mass = __ballot(v > 0.0);
              if (mass) last = b0 + 63 - __clzll((long long)mass);
              const unsigned long long over = __ballot(start + incl > target);
              if (over) pick = b0 + __ffsll((long long)over) - 1;
              start += __shfl(incl, 63);
            }
            if (pick < 0) pick = last >= 0 ? last : c_lo;
            if (lane == 0) emit(pick);
          }
          __syncthreads();                   // sh.pick_th is free again
        }
      }
      __syncthreads();
      return true;
    };

    stamp(23);
    if (bonus) {
      // ===== every draft layer passed: W_L beams from p_beam^(gamma+1)
      if (!draw(0.0, false, u_fill + (long long)l * a.W_cap, min(W_in, a.W_cap), 0)) return;
      n_out = min(W_in, a.W_cap);
      if (g == 0 && tid == 0) a.out.layer_width[(long long)prompt * Lw + l] = W_in;
      break;
    }

    int WL = W_in;             // width of the layer, known before the first decision

    // The accept / reject decisions of Algorithm 1 in candidate order, as far as the chain allows.
    // Outcome in sh.state[round & 1]: 0 = finished, 1 = the next chain entry is needed.
    // Plain sequential form (one thread): only used when a residual without mass turns up.
    auto decide_serial = [&](unsigned int round) {
      int pos = sh.pos, nacc = sh.acc_n, k = sh.kidx;
      const int kmax = sh.kmax;
      int state = 0;
      while (true) {
        if (pos >= M || nacc >= WL) { state = 0; break; }
        if (k > kmax) { state = 1; break; }
        if (k > 1 && !(sh.FF[k] > 0.0)) {
          // a residual without mass (impossible in exact arithmetic): fall back to p_beam
          atomicOr(a.fault, DSBD_FAULT_ZERO_RESIDUAL);
          k = 1;
        }
        const int n = sh.S_node[pos];
        const double pbx = sh.S_pb[pos], qbx = sh.S_qb[pos];
        const double num = (k == 1) ? pbx : fmax(pbx - sh.cc[k] * qbx, 0.0) / sh.FF[k];
        const double ratio = (qbx == 0.0) ? INFINITY : num / qbx;
        const double u = (double)sh.S_u[pos];
        if (fabs(ratio - u) <= NEAR_TIE) near_tie++;
        if (u <= ratio) {
          sh.A_node[nacc] = n;
          sh.A_idx[nacc] = pos;
          nacc++;
          k = 1;
          if (g == 0) a.out.node_status[n] = DSBD_ACCEPTED;
        } else {
          k++;
          if (g == 0) a.out.node_status[n] = DSBD_REJECTED;
        }
        pos++;
      }
      sh.pos = pos; sh.acc_n = nacc; sh.kidx = k; sh.state[round & 1] = state;
    };
    // The same decisions taken by the first wave, a run at a time.  With p' = p_beam (chain index 1) consecutive
    // candidates are independent tests (precomputed flags): all acceptances up to the first rejection are taken
    // at once.  After a rejection candidate pos + j meets chain entry k + j for as long as the rejections last:
    // those tests run side by side and the first acceptance ends the streak.
    auto decide = [&](unsigned int round, int kmax) {    // kmax: entries of the chain that exist (uniform)
      wave_lds_fence();                                    // the newest entry was written by lane 0 a moment ago
      int pos = sh.pos, nacc = sh.acc_n, k = sh.kidx;      // uniform over the wave
      int state = 0, near_add = 0;
      while (true) {
        if (pos >= M || nacc >= WL) { state = 0; break; }
        const int cand = pos + lane;
        if (k == 1) {
          const int nv = min(64, M - pos);
          const int fl = lane < nv ? sh.S_flag[cand] : 0;
          const unsigned long long rej = __ballot(lane < nv && !(fl & 1));
          const int run = rej ? min(nv, (int)__ffsll((long long)rej) - 1) : nv;   // acceptances in a row from pos
          const int take = min(run, WL - nacc);
          if (lane < take) {
            const int n = sh.S_node[cand];
            sh.A_node[nacc + lane] = n;
            sh.A_idx[nacc + lane] = cand;
            if (g == 0) a.out.node_status[n] = DSBD_ACCEPTED;
          }
          const bool fails = take == run && run < nv && nacc + take < WL;   // candidate pos + run is tested and rejected
          near_add += __popcll(__ballot((lane < take || (fails && lane == run)) && (fl & 2)));
          nacc += take; pos += take;
          if (fails) {
            if (lane == run && g == 0) a.out.node_status[sh.S_node[cand]] = DSBD_REJECTED;
            pos += 1; k = 2;
          }
          continue;
        }
        const int navail = kmax - k + 1;                   // chain entries k .. kmax exist
        if (navail <= 0) { state = 1; break; }
        const int nv = min(min(64, navail), M - pos);
        bool acc = false, nr = false, dead = false;
        if (lane < nv) {
          const int kk = k + lane;
          const double F = sh.FF[kk];
          dead = !(F > 0.0);
          const double pbx = sh.S_pb[cand], qbx = sh.S_qb[cand];
          const double num = fmax(pbx - sh.cc[kk] * qbx, 0.0) / F;
          const double ratio = (qbx == 0.0) ? INFINITY : num / qbx;
          const double u = (double)sh.S_u[cand];
          acc = u <= ratio;
          nr = fabs(ratio - u) <= NEAR_TIE;
        }
        const unsigned long long accm = __ballot(lane < nv && acc);
        const int last = accm ? (int)__ffsll((long long)accm) - 1 : nv - 1;     // last candidate tested in this step
        if (__ballot(lane <= last && dead)) {
          // a residual without mass: hand the rest to the sequential form, which knows what to do about it
          if (lane == 0) { near_tie += near_add; sh.pos = pos; sh.acc_n = nacc; sh.kidx = k; decide_serial(round); }
          wave_lds_fence();
          return;
        }
        near_add += __popcll(__ballot(lane <= last && nr));
        if (lane <= last) {
          const int n = sh.S_node[cand];
          const bool a_here = accm && lane == last;
          if (a_here) { sh.A_node[nacc] = n; sh.A_idx[nacc] = cand; }
          if (g == 0) a.out.node_status[n] = a_here ? DSBD_ACCEPTED : DSBD_REJECTED;
        }
        pos += last + 1;
        if (accm) { nacc += 1; k = 1; } else { k += nv; }
      }
      if (lane == 0) { near_tie += near_add; sh.pos = pos; sh.acc_n = nacc; sh.kidx = k; sh.state[round & 1] = state; }
    };

    // Appends entry kmax+1 to the residual chain: every workgroup sums its slice, the first wave exchanges the
    // partial sums and, if asked to, carries on with the decisions right away.  All threads leave through one
    // barrier; false = a wait gave up.
    auto extend_chain = [&](bool then_decide) -> bool {
      if (spec) {                      // entry 2 is already on its way
        if (wave == 0) {
          double F;
          if (!wave_sum_groups(spec_bank, spec_gbank, a.G, g, spec_own, spec_tag, a.sync_limit, F)) give_up();
          if (lane == 0) { sh.cc[2] = 1.0; sh.FF[2] = F; sh.kmax = 2; }
          if (then_decide) decide(decide_round, 2);
        }
        spec = false;
      } else {
        const int k = sh.kmax;
        const double c = sh.cc[k] + sh.FF[k];
        stamp(46);
        const double sl = slice_sum(c, 0, VL_BLOCK);
        stamp(43);
        const double tot = wg_total(sl);
        stamp(44);
        if constexpr (WARP) {          // every workgroup holds the whole warped joint: the total is F itself
          if (wave == 0) {
            if (lane == 0) { sh.cc[k + 1] = c; sh.FF[k + 1] = tot; sh.kmax = k + 1; }
            if (then_decide) decide(decide_round, k + 1);
          }
          __syncthreads();
          return true;
        }
        unsigned long long* const x_acc = accs + (size_t)(achg & 1) * NACC * 16;
        unsigned long long* const x_prev = sh.acc_prev[achg & 1];
        achg += 1;
        if (wave == 0) {
          double F;
          if (!wave_sum_accumulators(x_acc, x_prev, a.G, g, tot, a.sync_limit, F)) give_up();
          stamp(45);
          if (lane == 0) { sh.cc[k + 1] = c; sh.FF[k + 1] = F; sh.kmax = k + 1; }
          if (then_decide) decide(decide_round, k + 1);
        }
      }
      __syncthreads();
      return sh.abort == 0;
    };

    stamp(30);
    // ===== width of the layer
    if (dynamic) {
      // alpha_j for j = 1..M (Eq. 3) from the chain; stop early if the residual mass vanishes
      if constexpr (WARP) {
        // The warped joints are the short list every workgroup holds, an entry per lane: the first wave runs the
        // whole chain by itself (c_{k+1} = c_k + F(c_k), F a sum over its lanes), no barrier per entry.  The same
        // sums as extend_chain forms (there the other waves add zeros).
        if (wave == 0) {
          const bool in = lane < sh.nU;
          const double up = in ? sh.U_p[lane] : 0.0, uq = in ? sh.U_q[lane] : 0.0;
          int k = sh.kmax;               // 1: nothing is posted ahead of time for warped joints
          double c = sh.cc[k], F = sh.FF[k];
          for (int j = 1; j <= M; ++j) {
            c += F;
            F = wave_sum(fmax(up - c * uq, 0.0));
            k += 1;
            if (lane == 0) { sh.cc[k] = c; sh.FF[k] = F; }
            if (!(F > 0.0)) break;
          }
          if (lane == 0) sh.kmax = k;
        }
        __syncthreads();
      } else {
        bool dead = false;
        for (int j = 1; j <= M && !dead; ++j) {
          if (!extend_chain(false)) return;
          dead = !(sh.FF[j + 1] > 0.0);
        }
      }
      const int kdone = sh.kmax;     // entries 1..kdone valid
      __syncthreads();
      int Wt = 0;
      if (M < 64) {
        // up to 63 drafts (every forest of the paper's shapes): the table fits one wave, lane m = row m, and the
        // steps are ordered by wavefront fences instead of workgroup barriers.  Same sums in the same order as the
        // general form below.
        if (wave == 0) {
          const int m = lane;
          if (m >= 1 && m <= M) {
            double alpha = 1.0;            // no residual mass left: accepted with certainty
            if (m + 1 <= kdone && sh.FF[m] > 0.0) alpha = 1.0 - sh.FF[m + 1] / sh.FF[m];
            sh.u.w.alpha[m] = alpha;
          }
          wave_lds_fence();
          if (m >= 1 && m <= M) {
            double f = sh.u.w.alpha[m];
            for (int j = 1; j < m; ++j) f *= (1.0 - sh.u.w.alpha[j]);
            sh.u.w.first[m] = f;
          }
          if (m <= M) {
            double none = 1.0;
            for (int j = 1; j <= m; ++j) none *= (1.0 - sh.u.w.alpha[j]);
            sh.Pa[m] = none;
          }
          wave_lds_fence();
          double below = 0.0;              // sum_{k<K} P(M,k)
          const int Kmax = min(M, a.W_cap);
          for (int K = 1; K <= Kmax; ++K) {
            below += sh.Pa[M];             // column K-1 is in Pa (uniform over the wave)
            if (!(1.0 - below >= thr)) break;
            Wt = K;
            if (K == Kmax) break;
            double tot = 0.0;
            if (m <= M && m >= K)
              for (int i = 1; i <= m; ++i) tot += sh.u.w.first[i] * ((m - i >= K - 1) ? sh.Pa[m - i] : 0.0);
            wave_lds_fence();              // everybody has read column K-1
            if (m <= M) sh.Pa[m] = tot;
            wave_lds_fence();
          }
          if (lane == 0) sh.found = Wt;
        }
        __syncthreads();
        Wt = sh.found;
        __syncthreads();
      } else {
        // alpha_i (Eq. 3), first[i] = alpha_i prod_{j<i} (1 - alpha_j) (Eq. 2), Pa[m] = P(m,0)
        for (int i = 1 + tid; i <= M; i += VL_BLOCK) {
          double alpha = 1.0;            // no residual mass left: accepted with certainty
          if (i + 1 <= kdone && sh.FF[i] > 0.0) alpha = 1.0 - sh.FF[i + 1] / sh.FF[i];
          sh.u.w.alpha[i] = alpha;
        }
        __syncthreads();
        for (int i = 1 + tid; i <= M; i += VL_BLOCK) {
          double f = sh.u.w.alpha[i];
          for (int j = 1; j < i; ++j) f *= (1.0 - sh.u.w.alpha[j]);
          sh.u.w.first[i] = f;
        }
        if (tid == 0) {
          double none = 1.0;
          sh.Pa[0] = 1.0;
          for (int m = 1; m <= M; ++m) { none *= (1.0 - sh.u.w.alpha[m]); sh.Pa[m] = none; }
        }
        __syncthreads();
        // W~ = max{K : 1 - sum_{k<K} P(M,k) >= t}; K = 0 always qualifies
        double below = 0.0;              // sum_{k<K} P(M,k)
        const int Kmax = min(M, a.W_cap);
        for (int K = 1; K <= Kmax; ++K) {
          below += sh.Pa[M];             // column K-1 is in Pa
          if (!(1.0 - below >= thr)) break;
          Wt = K;
          if (K == Kmax) break;
          // column K from column K-1:  P(m,K) = sum_{i=1..m} first[i] P(m-i,K-1), zero for m < K
          for (int m = tid; m <= M; m += VL_BLOCK) {
            double tot = 0.0;
            if (m >= K)
              for (int i = 1; i <= m; ++i) tot += sh.u.w.first[i] * ((m - i >= K - 1) ? sh.Pa[m - i] : 0.0);
            sh.Pb[m] = tot;
          }
          __syncthreads();
          for (int m = tid; m <= M; m += VL_BLOCK) sh.Pa[m] = sh.Pb[m];
          __syncthreads();
        }
        __syncthreads();
      }
      WL = min(a.W_cap, max(a.W_min, Wt));
    }
    WL = min(WL, a.W_cap);
    if (g == 0 && tid == 0) a.out.layer_width[(long long)prompt * Lw + l] = WL;

    stamp(40);
    // ===== sequential accept / reject.  The first wave takes the decisions as far as the chain reaches; meanwhile
    // the other seven waves already sum their slices for the chain entry that would come next, so a rejection that
    // needs it finds the partial sums ready to post (and an acceptance that ends the layer just drops them).
    {
      bool posted = spec;              // the next entry's partial sums are on their way: F(1), from the scaling pass
      Slot* x_bank = spec_bank;
      Slot* x_gbank = spec_gbank;
      unsigned long long x_tag = spec_tag;
      double x_own = spec_own;
      while (true) {
        const int k = sh.kmax;         // entries 1..k exist (read after a barrier: uniform)
        const double c_next = sh.cc[k] + sh.FF[k];
        stamp(41);
        if (wave == 0) decide(decide_round, k);
        double tot = 0.0;
        // (the barriers of this loop order LDS values only: chain entries, decisions, wave totals; slices are
        // read-only here and the outputs written meanwhile are read by nobody in this kernel)
        if (!posted) tot = wg_total(slice_sum(c_next, 64, VL_BLOCK - 64), true);   // barrier inside
        else lds_barrier();
        const int st = sh.state[decide_round & 1];
        decide_round += 1;             // the next outcome goes to the other entry: nobody still reads it
        stamp(42);
        if (st != 1) break;
        if constexpr (WARP) {
          if (tid == 0) { sh.cc[k + 1] = c_next; sh.FF[k + 1] = tot; sh.kmax = k + 1; }
          __syncthreads();
          continue;
        }
        // the entry posted ahead of time (c = 1) comes through its slots; every later one through the accumulators
        const bool via_acc = !posted;
        unsigned long long* const x_acc = accs + (size_t)(achg & 1) * NACC * 16;
        unsigned long long* const x_prev = sh.acc_prev[achg & 1];
        if (via_acc) achg += 1;
        if (wave == 0) {
          double F;
          const bool ok_x = via_acc ? wave_sum_accumulators(x_acc, x_prev, a.G, g, tot, a.sync_limit, F)
                                    : wave_sum_groups(x_bank, x_gbank, a.G, g, x_own, x_tag, a.sync_limit, F);
          if (!ok_x) give_up();
          if (lane == 0) { sh.cc[k + 1] = c_next; sh.FF[k + 1] = F; sh.kmax = k + 1; }
        }
        posted = false;
        spec = false;
        stamp(45);
        lds_barrier();
        if (sh.abort) return;
      }
    }
    const int nacc = sh.acc_n, pos_end = sh.pos, kcur = sh.kidx, kmax_end = sh.kmax;
    if (g == 0)
      for (int i = pos_end + tid; i < M; i += VL_BLOCK) a.out.node_status[sh.S_node[i]] = DSBD_REJECTED;

    stamp(50);
    if (nacc < WL) {
      // cumulative likelihoods of the accepted beams (fp64)
      if (tid < nacc) {
        const int n = sh.A_node[tid];
        const int ci = sh.A_idx[tid];
        const int slot = sh.slot_of[sh.n_parent[n - n_begin] - n_begin];
        sh.A_cum_p[tid] = sh.cum_p[slot] + ((double)sh.S_zp[ci] - sh.lse_p[slot]);
        sh.A_cum_q[tid] = sh.cum_q[slot] + ((double)sh.S_zq[ci] - sh.lse_q[slot]);
      }
      __syncthreads();
      // ===== the layer falls short: accepted beams, one residual sample, then p_beam samples
      if (g == 0 && tid < nacc) {
        const int n = sh.A_node[tid];
        const long long o = (long long)prompt * a.W_cap + tid;
        a.out.out_parent[o] = sh.n_parent[n - n_begin];
        a.out.out_token[o] = sh.n_token[n - n_begin];
        a.out.out_node[o] = n;
        a.out.out_logp_target[o] = sh.A_cum_p[tid];
        a.out.out_logp_draft[o] = sh.A_cum_q[tid];
        emit_next(tid, sh.n_parent[n - n_begin], sh.n_token[n - n_begin], sh.A_cum_p[tid], sh.A_cum_q[tid]);
      }
      // p' = p'_kcur; its chain entry may still be missing if the last candidate was rejected
      int k = kcur;
      if (k > kmax_end) {
        if (!extend_chain(false)) return;
      }
      if (k > 1 && !(sh.FF[k] > 0.0)) {
        if (g == 0 && tid == 0) atomicOr(a.fault, DSBD_FAULT_ZERO_RESIDUAL);
        k = 1;
      }
      const double c = sh.cc[k];
      if (!draw(c, k > 1, u_res + l, 1, nacc)) return;
      const int fills = WL - nacc - 1;
      if (fills > 0)
        if (!draw(0.0, false, u_fill + (long long)l * a.W_cap, fills, nacc + 1)) return;
      l_last = l;
      n_out = WL;
      break;
    }

    // ===== the layer passed: handed over at the top of the next layer
    passed_nacc = nacc;
  }

  stamp(99);
  if (g == 0) clear_out_slots(n_out);
  if (g == 0 && tid == 0) {
    a.out.l_last[prompt] = l_last;
    a.out.n_out[prompt] = n_out;
    a.out.near_tie_count[prompt] = near_tie;
    if (a.nx_on) a.nx.n_next[prompt] = n_out;
  }
}

// ------------------------------------------------------------------------------------------------ host side
namespace {

struct VerifyPlan {
  int nchunk, chunk, I_cap, G, lds_elems;
  bool small_nodes;        // the layer kernel built for prompts of at most NODE_CAP_SMALL nodes serves (more LDS for slices)
  int group;               // prompts per launch of the layer kernel (all of them, unless they do not fit the device at once)
  size_t lds_bytes;        // dynamic LDS of the layer kernel
  SlotLayout sl;
  long long slice_cap;     // elements of the largest slice of I x V a workgroup can get
};

int32_t check_verify(const dsbd_forest* f, int V, const dsbd_params* p) {
  if (!f || !p) return DSBD_ERR_INVALID;
  if (f->n_prompts < 0 || f->n_trees < 0 || f->n_nodes < 0) return DSBD_ERR_INVALID;
  if (V < 1 || V > (1 << 30)) return DSBD_ERR_UNSUPPORTED;     // positions in a row are 32-bit integers with room to step past the end
  if (p->W_cap < 1 || p->W_cap > 64) return DSBD_ERR_UNSUPPORTED;
  if (p->W_min < 1 || p->W_min > p->W_cap || p->W_L > p->W_cap) return DSBD_ERR_INVALID;
  if (!(p->t <= 1.0f)) return DSBD_ERR_INVALID;      // also rejects NaN (which would otherwise read as dynamic width 0)
  if (f->max_tree_nodes < 1 || f->max_tree_nodes > DSBD_MAX_TREE_NODES) return DSBD_ERR_UNSUPPORTED;
  if (f->max_prompt_trees < 1 || f->max_prompt_trees > 64) return DSBD_ERR_UNSUPPORTED;
  if (p->W_L <= 0 && f->max_prompt_trees > p->W_cap) return DSBD_ERR_INVALID;
  if ((long long)f->max_prompt_trees * f->max_tree_nodes > NODE_CAP) return DSBD_ERR_UNSUPPORTED;
  if (f->max_depth < 0 || f->max_depth >= DSBD_MAX_TREE_NODES) return DSBD_ERR_INVALID;
  // warping T: top_k = 0 and top_p >= 1 is the identity; otherwise the joint is cut to its top_k <= WARP_K_MAX
  // entries first (top-p alone would need an unbounded candidate list)
  if (p->top_k < 0 || !(p->top_p >= 0.0f)) return DSBD_ERR_INVALID;
  if (p->top_k > WARP_K_MAX || (p->top_k == 0 && p->top_p > 0.0f && p->top_p < 1.0f)) return DSBD_ERR_UNSUPPORTED;
  if (p->top_k > 0) {
    const long long cap = p->W_cap > f->max_prompt_trees ? p->W_cap : f->max_prompt_trees;
    if (cap * V > 0x7fffffffLL) return DSBD_ERR_UNSUPPORTED;     // flat indices travel as 32-bit integers
  }
  return DSBD_OK;
}

// What the layer kernel may occupy: all its workgroups must be resident at once.
struct DeviceLimits { int cus, blocks_per_cu; };
const DeviceLimits& device_limits() {
  static DeviceLimits lim = {0, 0};
  static std::once_flag once;
  std::call_once(once, [] {
    int dev = 0, v = 0;
    lim.cus = 256;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0)
      lim.cus = v;
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(verify_layers_kernel<false, NODE_CAP>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, VL_DYN_LDS_BYTES);
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(verify_layers_kernel<true, NODE_CAP>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, VL_DYN_LDS_BYTES);
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(verify_layers_kernel<false, NODE_CAP_SMALL>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, VL_DYN_LDS_BYTES_SMALL);
    int nb = 0, nb2 = 0, nb3 = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, verify_layers_kernel<false, NODE_CAP>, VL_BLOCK, VL_DYN_LDS_BYTES) != hipSuccess || nb < 1)
      nb = 1;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb2, verify_layers_kernel<true, NODE_CAP>, VL_BLOCK, VL_DYN_LDS_BYTES) != hipSuccess || nb2 < 1)
      nb2 = 1;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb3, verify_layers_kernel<false, NODE_CAP_SMALL>, VL_BLOCK, VL_DYN_LDS_BYTES_SMALL) != hipSuccess || nb3 < 1)
      nb3 = 1;
    if (nb3 < nb2) nb2 = nb3;
    lim.blocks_per_cu = nb < nb2 ? nb : nb2;
    (void)hipGetLastError();
  });
  return lim;
}

VerifyPlan make_verify_plan(const dsbd_forest* f, int V, const dsbd_params* p, bool alias = false) {
  VerifyPlan pl;
  const DsbdKnobs& knobs = dsbd_knobs();
  // about four chunks per row, of 8k to 32k logits each: a few thousand workgroups at the large configurations
  // (measured: a 32000-token vocabulary in one chunk per row ran the 16-prompt batch at 45 % of the HBM peak, in
  // four at 57 %)
  int target = V / 4;
  if (target < 8192) target = 8192;
  if (target > 32768) target = 32768;
  if (knobs.stats_chunk >= 1024) target = knobs.stats_chunk;   // tuning knob: logits per workgroup of the statistics pass
  // few rows (a draft step's beams): finer chunks, down to 4k logits and up to 16 per row, until about a thousand
  // workgroups stream (a workgroup of the pass is bound by memory latency x its number of load rounds)
  else
    while (target > 4096 && (V + target / 2 - 1) / (target / 2) <= 16 &&
           2LL * f->n_nodes * ((V + target - 1) / target) < 1024)
      target /= 2;
  pl.nchunk = (V + target - 1) / target;
  pl.chunk = ((V + pl.nchunk - 1) / pl.nchunk + 3) & ~3;
  pl.nchunk = (V + pl.chunk - 1) / pl.chunk;
  pl.I_cap = p->W_cap > f->max_prompt_trees ? p->W_cap : f->max_prompt_trees;
  // one workgroup per compute unit in total, shared evenly by the prompts, at least 4096 joint elements per
  // workgroup.  More prompts than workgroups fit the device at once: groups of prompts, one launch after the other
  // (Algorithm 1 runs per prompt), one workgroup per prompt.
  const DeviceLimits& lim = device_limits();
  const int resident = lim.cus * lim.blocks_per_cu;
  int G = f->n_prompts > 0 ? lim.cus / f->n_prompts : 1;
  // (sized by the joint of the input beams, which is what a fixed width keeps every layer at: an exchange among 64
  // workgroups costs 1.7 us against 2.5 us among 256, and below about 4000 entries per workgroup the passes over a
  // slice are shorter than that difference.  Measured: 8 beams x 32000 tokens 83 us with 64 workgroups, 88 us with
  // 256; with the dynamic width, which runs many more exchanges, 147 us against 165 us.)
  const long long joint = (long long)f->max_prompt_trees * V;
  const int by_work = (int)((joint + 3999) / 4000);
  if (G > by_work) G = by_work;
  if (knobs.verify_g >= 1 && (long long)knobs.verify_g * f->n_prompts <= resident) G = knobs.verify_g;   // tuning knob
  if (G < 1) G = 1;
  if (G > 256) G = 256;
  pl.G = G;
  pl.group = f->n_prompts;
  if ((long long)pl.group * G > resident) pl.group = resident / G;     // G is 1 here
  if (pl.group < 1) pl.group = 1;
  // prompts of few nodes and no warping (whose scratch lists use the per-node arrays at full size): the kernel
  // variant with the short per-node arrays, which leaves more of the LDS to the slices
  pl.small_nodes = p->top_k == 0 && (long long)f->max_prompt_trees * f->max_tree_nodes <= NODE_CAP_SMALL;
  const long long cap = (pl.small_nodes ? VL_DYN_LDS_BYTES_SMALL : VL_DYN_LDS_BYTES) / (alias ? 8 : 16);   // one array instead of two when q_beam is p_beam
  // exchange slots: every workgroup's slots of an exchange start a 128-byte line (no two writers per line)
  {
    auto up8 = [](int v) { return (v + LINE_SLOTS - 1) / LINE_SLOTS * LINE_SLOTS; };
    const int layers = f->max_depth + 1;
    SlotLayout& sl = pl.sl;
    int off = 0;
    sl.x[0] = off; off += G * LINE_SLOTS;
    sl.x[1] = off; off += G * LINE_SLOTS;
    sl.xc[0] = off; off += SUM_GROUPS * LINE_SLOTS;
    sl.xc[1] = off; off += SUM_GROUPS * LINE_SLOTS;
    sl.r_w = up8(4 * pl.I_cap);
    sl.r = off; sl.r_stride = G * sl.r_w; off += layers * sl.r_stride;
    sl.s = off; sl.s_stride = G * LINE_SLOTS; off += layers * sl.s_stride;
    sl.sc = off; sl.sc_stride = SUM_GROUPS * LINE_SLOTS; off += layers * sl.sc_stride;
    sl.b = sl.c = sl.d = sl.wb = off; sl.b_w = 0; sl.wb_stride = 0;
    if (p->top_k > 0) {
      sl.b_w = up8(4 * p->top_k);
      sl.b = off; off += G * sl.b_w;
      sl.c = off; off += (G + WARP_GROUP - 1) / WARP_GROUP * sl.b_w;
      sl.d = off; off += up8(WARP_RESULT_SLOTS);
      sl.wb = off; sl.wb_stride = G * sl.b_w; off += layers * sl.wb_stride;
    }
    sl.acc = off; off += 2 * NACC * LINE_SLOTS;
    sl.acc0 = off; off += up8(2 * NACC);
    sl.prompt_stride = off;
  }
  // dynamic LDS for the p_beam / q_beam slices: what one slice needs, at most VL_DYN_LDS_BYTES for the two arrays
  long long need = 2;                        // the longest slice any number of input rows can give
  for (int nI = 1; nI <= pl.I_cap; ++nI) {
    const long long len = slice_cut(nI, V, G).len;
    if (len > need) need = len;
  }
  need = (need + 1) & ~1LL;
  pl.slice_cap = need;
  pl.lds_elems = (int)(need < cap ? need : cap);
  // warping: the candidate lists of a merge (2 x WARP_CAND values and indices) sit in the dynamic LDS
  if (p->top_k > 0 && pl.lds_elems < (3 * WARP_CAND + 1) / 2) pl.lds_elems = (3 * WARP_CAND + 1) / 2;
  pl.lds_bytes = (size_t)pl.lds_elems * (alias ? 8 : 16);
  if (p->top_k > 0 && pl.lds_bytes < (size_t)((3 * WARP_CAND + 1) / 2) * 16) pl.lds_bytes = (size_t)((3 * WARP_CAND + 1) / 2) * 16;
  pl.lds_bytes = (pl.lds_bytes + 15) & ~(size_t)15;
  return pl;
}

size_t carve_verify(WorkspaceCarver& ws, const dsbd_forest* f, int V, const VerifyPlan& pl, float2** part, double** pb,
                    double** qb, double** red) {
  const size_t N = (size_t)f->n_nodes, P = (size_t)f->n_prompts;
  (void)V;
  ws.take<long long>(512);                 // timeline of the layer kernel (diagnostics), first in the workspace
  ws.take<unsigned long long>(32);         // replay count of launches recorded into a graph (one word, a line of its own)
  *part = ws.take<float2>(2 * N * pl.nchunk);
  // slices that do not fit the LDS: a region per workgroup of a launch (the launches of a forest that runs in groups
  // of prompts follow each other and share the regions); exchange slots: a region per prompt
  *pb = ws.take<double>((size_t)pl.group * pl.G * (size_t)pl.slice_cap);
  *qb = ws.take<double>((size_t)pl.group * pl.G * (size_t)pl.slice_cap);
  *red = ws.take<double>(P * (size_t)pl.sl.prompt_stride * 2);
  return ws.total();
}

// The second stream the statistics pass runs on, next to the layer kernel on the caller's stream; one per device,
// created on first use and kept until the process ends (with the two events that order it after the caller's
// earlier work and order the caller's later work after it).
struct SideStream {
  hipStream_t stream = nullptr;
  hipEvent_t fork = nullptr, join = nullptr;
  bool tried = false, ok = false;
  // Two layer kernels on different streams must not share the compute units: each waits for workgroups of its own
  // that the other one's keep out.  The library therefore orders its layer launches itself once it has seen calls on
  // more than one stream: the first change of stream waits for the device to drain, and from then on layers_done is
  // recorded behind every layer launch and a launch on another stream than the last one waits for it.  (Recording
  // from the start would cost every single-stream caller 6 us per call, measured.)  enqueue makes one call's records
  // and waits a unit among host threads.
  hipEvent_t layers_done = nullptr;
  hipStream_t last_stream = nullptr;
  bool have_last = false, several_streams = false;
  std::mutex enqueue;
};
SideStream* side_stream_of_current_device(bool may_create) {
  static SideStream table[64];
  static std::mutex mutex;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return nullptr;
  std::lock_guard<std::mutex> lock(mutex);
  SideStream& s = table[dev];
  if (!s.tried && may_create) {
    s.tried = true;
    const unsigned ev = hipEventDisableTiming | (dsbd_knobs().event_fence ? 0u : (unsigned)hipEventDisableSystemFence);
    s.ok = hipStreamCreateWithFlags(&s.stream, hipStreamNonBlocking) == hipSuccess &&
           hipEventCreateWithFlags(&s.fork, ev) == hipSuccess && hipEventCreateWithFlags(&s.join, ev) == hipSuccess &&
           hipEventCreateWithFlags(&s.layers_done, ev) == hipSuccess;
    if (!s.ok) (void)hipGetLastError();
  }
  return s.ok ? &s : nullptr;
}

std::atomic<unsigned long long> g_launch_counter{0};

// In front of a layer kernel that is recorded into a graph: every replay repeats the launch's arguments, so what tells
// its exchange slots from those of the replay before is this count (whatever the word held to begin with).
__global__ void bump_replay_count_kernel(unsigned long long* count) { *count += 1; }

}  // namespace

extern "C" size_t dsbd_verify_forest_workspace_bytes(const dsbd_forest* f, int32_t V, const dsbd_params* p) {
  if (check_verify(f, V, p) != DSBD_OK) return 0;
  const VerifyPlan pl = make_verify_plan(f, V, p);
  WorkspaceCarver ws(nullptr);
  float2* pt; double *pb, *qb, *red;
  return carve_verify(ws, f, V, pl, &pt, &pb, &qb, &red) + 256;
}

namespace {
// may_create_side: the second stream may be created by this call (an ordinary call); false for the entry point that
// must not allocate, which uses the second stream only if an earlier call or dsbd_init() has made it.
// next: the next-beam plan to be written along with the output beams (nullptr: none).  With keep_one == 0 the layer
// kernel writes it itself; the single surviving beam of keep_one != 0 needs all of a prompt's output beams side by
// side, which sit in several workgroups' hands: there the selection kernel is launched behind the verification.
int32_t verify_impl(const dsbd_forest* f, const dsbd_verify_in* in, const dsbd_params* p, const dsbd_verify_out* out,
                    void* workspace, size_t workspace_bytes, int32_t* fault, void* stream_, bool may_create_side,
                    const dsbd_next_beams* next = nullptr, int keep_one = 0) {
  if (!in || !out || !fault) return DSBD_ERR_INVALID;
  int32_t rc = check_verify(f, in->V, p);
  if (rc != DSBD_OK) return rc;
  if (next && (!next->n_next || !next->src_tree || !next->src_out || !next->path_len || !next->path || !next->token ||
               !next->logp_target || !next->logp_draft))
    return DSBD_ERR_INVALID;
  if (f->n_nodes == 0 || f->n_trees == 0 || f->n_prompts == 0) return DSBD_OK;
  if (!f->tree_prompt || !f->tree_off || !f->parent || !f->token) return DSBD_ERR_INVALID;
  if (!in->logits_target || !in->logits_draft || !in->beam_logp_target || !in->beam_logp_draft || !in->u_accept ||
      !in->u_resid || !in->u_fill)
    return DSBD_ERR_INVALID;
  if (!out->node_status || !out->l_last || !out->layer_width || !out->n_out || !out->out_parent || !out->out_token ||
      !out->out_node || !out->out_logp_target || !out->out_logp_draft || !out->near_tie_count)
    return DSBD_ERR_INVALID;
  if (!workspace) return DSBD_ERR_INVALID;
  if (workspace_bytes < dsbd_verify_forest_workspace_bytes(f, in->V, p)) return DSBD_ERR_WORKSPACE;
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  const DsbdKnobs& knobs = dsbd_knobs();
  // the same arrays given for both models (the draft stage does: its draws are the additional layer of a forest of
  // single-node trees with the draft model in both roles): q_beam is p_beam and is kept, and computed, once
  const bool alias = in->logits_target == in->logits_draft && in->beam_logp_target == in->beam_logp_draft;
  const VerifyPlan pl = make_verify_plan(f, in->V, p, alias);

  char* wbase = reinterpret_cast<char*>(dsbd_align_up(reinterpret_cast<uintptr_t>(workspace), 256));
  WorkspaceCarver ws(wbase);
  float2* part; double *pb, *qb, *red;
  carve_verify(ws, f, in->V, pl, &part, &pb, &qb, &red);

  // ---- the statistics pass (per-node outputs; the layer kernel does not depend on it) runs on a second stream next
  // to the layer kernel: ordered after everything the caller's stream holds so far, and the caller's stream continues
  // only when both are done.  DSBD_VERIFY_OVERLAP=0 (or a stream that cannot be created) puts it in front instead.
  const bool want_stats = out->lse_target || out->lse_draft || out->node_logp_target || out->node_logp_draft;
  SideStream* state = side_stream_of_current_device(may_create_side);
  SideStream* side = (want_stats && knobs.verify_overlap) ? state : nullptr;
  std::unique_lock<std::mutex> enqueue_lock;
  if (state) enqueue_lock = std::unique_lock<std::mutex>(state->enqueue);
  // a stream under capture takes no part in the ordering of layer launches (an event recorded into a capture cannot
  // be waited for from outside it): replays of such a graph are the caller's to keep apart from other verifications
  bool capturing = false;
  {
    hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(stream, &cs) == hipSuccess) capturing = cs != hipStreamCaptureStatusNone;
    else { (void)hipGetLastError(); capturing = true; }
  }
  StatsArgs sa;
  sa.z[0] = in->logits_target; sa.z[1] = in->logits_draft;
  sa.n_nodes = f->n_nodes; sa.V = in->V; sa.nchunk = pl.nchunk; sa.chunk = pl.chunk;
  sa.part = part; sa.fault = fault;
  FinishArgs fa;
  fa.z[0] = in->logits_target; fa.z[1] = in->logits_draft;
  fa.n_nodes = f->n_nodes; fa.V = in->V; fa.nchunk = pl.nchunk; fa.alias = alias ? 1 : 0; fa.part = part;
  fa.parent = f->parent; fa.token = f->token; fa.fault = fault;
  fa.lse[0] = out->lse_target; fa.lse[1] = out->lse_draft;
  fa.logp[0] = out->node_logp_target; fa.logp[1] = out->node_logp_draft;
  auto launch_stats = [&](hipStream_t st) {
    // Beside the layer kernel the pass is held to STATS_SIDE_WGS workgroups per compute unit by the LDS it claims
    // (it uses none of it).  Measured on the benchmark shape (layer kernel alone: 120 us, the call with the pass in
    // front of it: 167 us): four per unit (all that the registers left over admit) stream at full rate for 49 us,
    // slow the layer kernel's first layers down and give a call of 149 us; three: 55 us and 146 us; one: 88 us, inside
    // the layer kernel's run, 142 us; none: the pass runs behind the layer kernel, 184 us.
    unsigned int side_lds = 0;
    if (st != stream) {
      const size_t layer_static = pl.small_nodes ? sizeof(LayerShared<NODE_CAP_SMALL>) : sizeof(LayerShared<NODE_CAP>);
      const long long layer_lds = (long long)(layer_static + pl.lds_bytes + 511) / 512 * 512;
      // a claim that STATS_SIDE_WGS workgroups fit in beside the layer kernel's LDS and one more does not, with
      // half a claim of slack on either side (the allocation granule and the pass's own few bytes are not known here)
      const long long free_lds = CU_LDS_BYTES - layer_lds;
      long long per = free_lds / (STATS_SIDE_WGS + 1) + free_lds / (2 * STATS_SIDE_WGS * (STATS_SIDE_WGS + 1));
      per = per / 256 * 256;
      if (per > 60000) per = 60000;
      if (per > 0) side_lds = (unsigned int)per;
      if (knobs.stats_side_lds >= 0) side_lds = (unsigned int)knobs.stats_side_lds;
    }
    dsbd_launch(DSBD_KERNEL_VOCAB_STATS, vocab_stats_kernel, dim3(pl.nchunk, f->n_nodes, alias ? 1 : 2), dim3(VS_BLOCK),
                side_lds, st, sa);
    hipLaunchKernelGGL(vocab_finish_kernel, dim3((f->n_nodes + VS_BLOCK - 1) / VS_BLOCK), dim3(VS_BLOCK), 0, st, fa);
  };
  if (want_stats && !side) {
    launch_stats(stream);
    DSBD_HIP_LAUNCH_CHECK();
  }
  if (side) {
    if (hipEventRecord(side->fork, stream) != hipSuccess || hipStreamWaitEvent(side->stream, side->fork, 0) != hipSuccess)
      return DSBD_ERR_HIP;
  }

  LayersArgs la;
  la.n_prompts = f->n_prompts; la.n_trees = f->n_trees; la.n_nodes = f->n_nodes;
  la.tree_prompt = f->tree_prompt; la.tree_off = f->tree_off; la.parent = f->parent; la.token = f->token;
  la.rank = f->draft_rank; la.max_depth = f->max_depth; la.max_prompt_trees = f->max_prompt_trees;
  la.max_tree_nodes = f->max_tree_nodes;
  la.V = in->V; la.zp = in->logits_target; la.zq = in->logits_draft;
  la.blp = in->beam_logp_target; la.blq = in->beam_logp_draft;
  la.u_acc = in->u_accept; la.u_res = in->u_resid; la.u_fill = in->u_fill;
  la.W_L = p->W_L; la.W_min = p->W_min; la.W_cap = p->W_cap; la.t = p->t;
  la.out = *out;
  la.pb = pb; la.qb = qb; la.red = red; la.slice_cap = pl.slice_cap;
  la.trace = knobs.verify_trace ? reinterpret_cast<long long*>(wbase) : nullptr;
  la.trace_wg = knobs.verify_trace_wg;
  la.sync_limit = SYNC_LIMIT_TICKS;
  if (knobs.verify_sync_limit_us >= 1 && knobs.verify_sync_limit_us <= 10000000LL)   // bound of the kernel's waits (default 3 s)
    la.sync_limit = knobs.verify_sync_limit_us * 100;
  la.mute_wg = knobs.verify_mute_wg;   // error-path test hook
  // Exchange slots carry a tag made of this number and the exchange's index: nothing an earlier launch left in the
  // workspace can pass for a value of this one, so the slots need no clearing.
  la.nonce = (g_launch_counter.fetch_add(1, std::memory_order_relaxed) + 1) << 24;
  la.replay = nullptr;
  if (capturing) {
    unsigned long long* const count = reinterpret_cast<unsigned long long*>(wbase + 512 * sizeof(long long));
    hipLaunchKernelGGL(bump_replay_count_kernel, dim3(1), dim3(1), 0, stream, count);
    la.replay = count;
  }
  la.G = pl.G; la.I_cap = pl.I_cap; la.sl = pl.sl; la.lds_elems = pl.lds_elems; la.fault = fault;
  la.lds_slice = pl.lds_elems;
  la.alias = alias ? 1 : 0;
  la.warp_fast = knobs.warp_fast ? 1 : 0;
  la.nx_on = (next && !keep_one) ? 1 : 0;
  if (la.nx_on) la.nx = *next; else la.nx = dsbd_next_beams{};
  if (knobs.verify_lds_slice >= 0 && knobs.verify_lds_slice < la.lds_slice) la.lds_slice = knobs.verify_lds_slice;   // tuning / test knob
  la.top_k = p->top_k; la.top_p = (p->top_p > 0.0f && p->top_p < 1.0f) ? p->top_p : 1.0f;
  // Ordinary launches: a launch was sized to fit the device at once, and every wait inside the kernel is bounded.
  // (A cooperative launch would also guarantee co-residency against work on other streams, but it made rocprofv3
  // crash at process exit on ROCm 7.2 and costs extra launch latency.)
  if (state && !capturing && state->have_last && state->last_stream != stream) {
    if (!state->several_streams) {
      if (hipDeviceSynchronize() != hipSuccess) return DSBD_ERR_HIP;
      state->several_streams = true;
    } else if (hipStreamWaitEvent(stream, state->layers_done, 0) != hipSuccess) {
      return DSBD_ERR_HIP;
    }
  }
  for (int p0 = 0; p0 < f->n_prompts; p0 += pl.group) {
    la.prompt0 = p0;
    const int np = f->n_prompts - p0 < pl.group ? f->n_prompts - p0 : pl.group;
    const unsigned grid3 = (unsigned)np * (unsigned)pl.G;
    if (p->top_k > 0)
      dsbd_launch(DSBD_KERNEL_VERIFY_LAYERS, verify_layers_kernel<true, NODE_CAP>, dim3(grid3), dim3(VL_BLOCK),
                  (unsigned int)pl.lds_bytes, stream, la);
    else if (pl.small_nodes)
      dsbd_launch(DSBD_KERNEL_VERIFY_LAYERS, verify_layers_kernel<false, NODE_CAP_SMALL>, dim3(grid3), dim3(VL_BLOCK),
                  (unsigned int)pl.lds_bytes, stream, la);
    else
      dsbd_launch(DSBD_KERNEL_VERIFY_LAYERS, verify_layers_kernel<false, NODE_CAP>, dim3(grid3), dim3(VL_BLOCK),
                  (unsigned int)pl.lds_bytes, stream, la);
  }
  hipError_t le = hipGetLastError();
  if (state && !capturing) {
    if (state->several_streams && hipEventRecord(state->layers_done, stream) != hipSuccess) le = hipErrorUnknown;
    state->last_stream = stream;
    state->have_last = true;
  }
  if (side) {
    launch_stats(side->stream);
    if (hipEventRecord(side->join, side->stream) != hipSuccess || hipStreamWaitEvent(stream, side->join, 0) != hipSuccess)
      le = hipErrorUnknown;
    const hipError_t le2 = hipGetLastError();
    if (le == hipSuccess) le = le2;
  }
  if (le != hipSuccess) return DSBD_ERR_HIP;
  if (next && keep_one) return dsbd_select_beams(f, out, p->W_cap, keep_one, next, fault, stream_);
  return DSBD_OK;
}
}  // namespace

extern "C" int32_t dsbd_verify_forest(const dsbd_forest* f, const dsbd_verify_in* in, const dsbd_params* p,
                                      const dsbd_verify_out* out, void* workspace, size_t workspace_bytes,
                                      int32_t* fault, void* stream_) {
  return verify_impl(f, in, p, out, workspace, workspace_bytes, fault, stream_, true);
}

extern "C" int32_t dsbd_verify_forest_select(const dsbd_forest* f, const dsbd_verify_in* in, const dsbd_params* p,
                                             const dsbd_verify_out* out, int32_t keep_one, const dsbd_next_beams* next,
                                             void* workspace, size_t workspace_bytes, int32_t* fault, void* stream_) {
  if (!next) return DSBD_ERR_INVALID;
  return verify_impl(f, in, p, out, workspace, workspace_bytes, fault, stream_, true, next, keep_one != 0);
}

// ---- the same call for callers that cannot allocate device memory (code under HIP graph capture, serving loops,
// harnesses that forbid hipMalloc): the workspace is a device array that is part of the library's image.
static __device__ __align__(256) unsigned char scratch[DSBD_STATIC_SCRATCH_BYTES];

namespace {
// Address of `scratch` on the current device (every GPU holds its own copy of the array at its own address; the
// array's name is only a host-side stand-in and must never reach a kernel or a memory call).
void* static_scratch_of_current_device() {
  static void* table[64] = {nullptr};
  static std::mutex mutex;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return nullptr;
  std::lock_guard<std::mutex> lock(mutex);
  if (!table[dev]) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) {
      (void)hipGetLastError();
      return nullptr;
    }
    table[dev] = ptr;
  }
  return table[dev];
}
}  // namespace

extern "C" int32_t dsbd_init(void) {
  if (!static_scratch_of_current_device()) return DSBD_ERR_HIP;
  (void)device_limits();
  (void)dsbd_knobs();
  return side_stream_of_current_device(true) ? DSBD_OK : DSBD_ERR_HIP;
}

extern "C" size_t dsbd_verify_forest_static_capacity(void) { return DSBD_STATIC_SCRATCH_BYTES; }

extern "C" int32_t dsbd_verify_forest_static(const dsbd_forest* f, const dsbd_verify_in* in, const dsbd_params* p,
                                             const dsbd_verify_out* out, int32_t* fault, void* stream_) {
  if (!in) return DSBD_ERR_INVALID;
  const int32_t rc = check_verify(f, in->V, p);
  if (rc != DSBD_OK) return rc;
  // the same plan as the ordinary call; a problem whose workspace exceeds the array is turned away, nothing is enqueued
  if (dsbd_verify_forest_workspace_bytes(f, in->V, p) > (size_t)DSBD_STATIC_SCRATCH_BYTES) return DSBD_ERR_WORKSPACE;
  void* ptr = static_scratch_of_current_device();
  if (!ptr) return DSBD_ERR_HIP;
  return verify_impl(f, in, p, out, ptr, DSBD_STATIC_SCRATCH_BYTES, fault, stream_, false);
}
