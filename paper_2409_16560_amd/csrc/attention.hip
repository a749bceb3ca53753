// Forest attention for gfx950 (paper Section 3.3, "Forest-based Parallel Decoding").
//
// Every node of tree b attends to beam b's prefix cache plus the tree rows of its ancestors and
// itself.  All nodes of a tree (times the query heads of one KV group) share one pass over the
// beam's K/V stream, which is what makes the step bandwidth-bound instead of re-reading the cache
// once per node.
//
// Work decomposition (split-KV): one workgroup per (tree, KV head, row block, KV split).  Inside a
// workgroup the 4 waves form RW row groups x TW token groups.  Every wave streams its own 32-token
// steps of K and V straight from HBM into registers (no block-level barrier in the main loop) and
// keeps 16*NRT query rows resident:
//   S^T = K Q^T   MFMA 16x16x32 bf16, A = K (tokens x d) from global in operand layout,
//                 B = Q^T held in registers for the whole kernel;
//   online softmax per query row, entirely lane-local: in the transposed product every lane owns
//                 one query row (column l%16), its scores and its slice of the output accumulators;
//   O^T += V^T P^T  MFMA 16x16x32, B = P^T built in registers from the S^T tile, A = V^T read from a
//                 wave-private LDS tile into which V was written transposed (token pairs packed).
// The ancestor mask never exists in memory: every wave derives the tree's topology itself (the parent array of
// a tree is one load per lane, the parent chains are walked with lane shuffles), each lane keeps the 64-bit
// ancestor bitmap of its row's node and tests bits while handling the (at most two) steps that cover the
// tree's own rows.  The first workgroup of a tree also reports what the walk found wrong with the parent array.
// Partial (m, l, O) of the KV splits go to the workspace; a second kernel merges them.
#include "common.h"
#include "topology_device.h"
#include <stdlib.h>

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float floatx4;
typedef short v4i16 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) v4i16 lds_v4i16;

#define NEG_BIG (-1.0e30f)
#define REF_SLACK 40.0f          // log2 headroom of the softmax reference before it is raised
#define STEP 32                 // tokens per wave step (two 16-token MFMA tiles)
#define VT_PITCH 36             // bf16 elements per row of the transposed V tile (32 + pad, multiple of 4)

struct AttnArgs {
  const int32_t* tree_off;
  const int32_t* parent;
  int max_tree_nodes, max_depth;
  uint64_t* anc_out;            // [n_nodes] ancestor-or-self bitmaps, written once per tree if not null
  const void* const* k_ptr;
  const void* const* v_ptr;
  const int32_t* len;
  const void* const* k_shared_ptr;
  const void* const* v_shared_ptr;
  const int32_t* shared_len;
  long long token_stride, head_stride;
  const __bf16* q;
  const __bf16* k_tree;
  const __bf16* v_tree;
  int n_nodes, Hq, Hkv, group;
  float scale_log2;             // scale * log2(e): scores are kept in the log2 domain
  int nsplit, n_rowblocks, max_len;
  float* part_o;                // [nsplit][n_nodes*Hq][D]
  float* part_ml;               // [nsplit][n_nodes*Hq][2]
  int32_t* fault;
  long long* trace;             // optional timeline of workgroup 0 (diagnostics): pairs (label, wall clock)
};

// 16-byte load through the GLOBAL address space.  The cache pointers come out of a pointer table in
// memory, so the compiler only knows them as generic pointers and would emit FLAT loads, which count on
// the LDS counter as well: every wait for an LDS read would then also wait for all K/V loads in flight.
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 load_global_16(const void* p) {
  const u32x4 v = *(const __attribute__((address_space(1))) u32x4*)(p);
  return make_uint4(v.x, v.y, v.z, v.w);
}
// The same with the non-temporal hint, for data that one thread consumes whole with one load (the K/V tiles of
// the shared-tile kernel: 9 % faster inside the benchmark's kernel mix).  Where a cache line is consumed by several
// load instructions of a wave (K in operand layout, wave-private kernel) the hint costs 20 % instead.
__device__ __forceinline__ uint4 load_global_16_nt(const void* p) {
  const u32x4 v = __builtin_nontemporal_load((const __attribute__((address_space(1))) u32x4*)(p));
  return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ bf16x8 load_global_bf16x8(const void* p) {
  union { uint4 u; bf16x8 v; } c;
  c.u = load_global_16(p);
  return c.v;
}

__device__ __forceinline__ void wave_lds_fence() {
  // orders this wave's LDS writes before its later LDS reads (other lanes' data); LDS executes a
  // wave's operations in order, so only the compiler needs to be held back
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Workgroup barrier that orders LDS traffic only.  __syncthreads() carries a workgroup-scope fence, for
// which the compiler waits for ALL outstanding memory operations (vmcnt(0)) - including the K/V loads of
// the next tile that were issued on purpose before the barrier, which would then never overlap with the
// arithmetic.  Here only the LDS counter is drained; global loads stay in flight across the barrier.
__device__ __forceinline__ void lds_barrier() {
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

template <int D, int NRT, int RW, int TW>
__global__ __launch_bounds__(256) void forest_attention_kernel(AttnArgs a) {
  static_assert(RW * TW == 4, "four waves per workgroup");
  constexpr int DS = D / 32;        // MFMA k-steps over the head dimension for S^T
  constexpr int DT = D / 16;        // 16-row output tiles over the head dimension for O^T
  constexpr int ROWS_W = 16 * NRT;  // query rows per wave
  constexpr int ROWS_B = ROWS_W * RW;
  constexpr int LPR = D / 8;        // lanes covering one V row with 16-byte loads
  constexpr int TG = 64 / LPR;      // token groups among the lanes for V loads
  constexpr int VROUNDS = STEP / (2 * TG);

  __shared__ __attribute__((aligned(16))) __bf16 vt_lds[4][D * VT_PITCH];
  __shared__ __attribute__((aligned(16))) float comb_o[(TW - 1) * RW][ROWS_W][D + 4];
  __shared__ float comb_ml[(TW - 1) * RW][ROWS_W][2];

  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int rw = wave % RW;
  const int tw = wave / RW;
  const int col = lane & 15;        // query row within a 16-row tile / token within a 16-token tile
  const int qd = lane >> 4;         // lane group 0..3

  int bid = blockIdx.x;
  const int split = bid % a.nsplit; bid /= a.nsplit;
  const int rb = bid % a.n_rowblocks; bid /= a.n_rowblocks;
  const int g = bid % a.Hkv;
  const int b = bid / a.Hkv;

  const dsbd_tree_range tr = dsbd_tree_range_of(b, a.n_nodes, a.tree_off, a.max_tree_nodes);
  const bool reporter = split == 0 && rb == 0 && g == 0 && wave == 0;   // one wave per tree speaks for it
  if (!tr.valid) {
    if (reporter && lane == 0) atomicOr(a.fault, tr.bad);
    return;
  }
  const int base = tr.base;
  const int n_b = min(tr.n_all, DSBD_MAX_TREE_NODES);
  const int p_mine = dsbd_tree_parent_of(tr, lane, a.parent);   // used once the first loads are on their way
  const int R = n_b * a.group;       // query rows of this (tree, KV head)
  const int row0 = rb * ROWS_B + rw * ROWS_W;
  const int n_rows_total = a.n_nodes * a.Hq;

  // ---- segments of the key sequence: shared prefix, own prefix, the tree's own rows
  int Ls = (a.shared_len && a.k_shared_ptr) ? a.shared_len[b] : 0;
  int Lo = a.len[b];
  Ls = max(Ls, 0); Lo = max(Lo, 0);
  int bad = 0;
  if ((long long)Ls + Lo > a.max_len) { bad |= DSBD_FAULT_BOUNDS; Ls = min(Ls, a.max_len); Lo = min(Lo, a.max_len - Ls); }
  const long long hoff = (long long)g * a.head_stride;
  const __bf16* k0 = Ls ? (const __bf16*)a.k_shared_ptr[b] : nullptr;
  const __bf16* v0 = Ls ? (const __bf16*)a.v_shared_ptr[b] : nullptr;
  const __bf16* k1 = Lo ? (const __bf16*)a.k_ptr[b] : nullptr;
  const __bf16* v1 = Lo ? (const __bf16*)a.v_ptr[b] : nullptr;
  if (Ls && (!k0 || !v0 || (((uintptr_t)k0 | (uintptr_t)v0) & 15))) { bad |= DSBD_FAULT_BOUNDS; Ls = 0; }
  if (Lo && (!k1 || !v1 || (((uintptr_t)k1 | (uintptr_t)v1) & 15))) { bad |= DSBD_FAULT_BOUNDS; Lo = 0; }
  if (bad && threadIdx.x == 0) atomicOr(a.fault, bad);   // missing or misaligned cache pointer: segment skipped
  k0 += hoff; v0 += hoff; k1 += hoff; v1 += hoff;
  const __bf16* k2 = a.k_tree + ((long long)base * a.Hkv + g) * D;
  const __bf16* v2 = a.v_tree + ((long long)base * a.Hkv + g) * D;
  const long long stride2 = (long long)a.Hkv * D;
  const int n0 = (Ls + STEP - 1) / STEP;
  const int n1 = (Lo + STEP - 1) / STEP;
  const int n2 = (n_b + STEP - 1) / STEP;
  const int total_steps = n0 + n1 + n2;
  // balanced partition: the first (total % nsplit) splits take one step more than the others
  const int st_begin = split * (total_steps / a.nsplit) + min(split, total_steps % a.nsplit);
  const int st_end = st_begin + total_steps / a.nsplit + (split < total_steps % a.nsplit ? 1 : 0);

  // ---- resident query fragments (B operand: lane holds row `col`, 8 channels 32j + 8qd ..)
  bf16x8 qf[NRT][DS];
  uint64_t anc[NRT];
#pragma unroll
  for (int rt = 0; rt < NRT; ++rt) {
    const int r = row0 + rt * 16 + col;
    const bool live = r < R;
    const int node = live ? r / a.group : 0;
    const int head = g * a.group + (live ? r % a.group : 0);
    anc[rt] = 0ull;
    const __bf16* qp = a.q + ((long long)(base + node) * a.Hq + head) * D + 8 * qd;
#pragma unroll
    for (int j = 0; j < DS; ++j) {
      if (live) {
        qf[rt][j] = load_global_bf16x8(qp + 32 * j);
      } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) qf[rt][j][e] = (__bf16)0.0f;
      }
    }
  }

  floatx4 o[NRT][DT];
  float m_run[NRT], l_run[NRT];
#pragma unroll
  for (int rt = 0; rt < NRT; ++rt) {
    m_run[rt] = NEG_BIG;
    l_run[rt] = 0.f;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) o[rt][dt] = floatx4{0.f, 0.f, 0.f, 0.f};
  }

  __bf16* vt = vt_lds[wave];
  const int v_dl = lane % LPR;       // 16-byte column of the V row this lane loads
  const int v_tg = lane / LPR;       // token group

  // a row block beyond the tree's rows has nothing to do (uniform over the workgroup)
  const bool block_live = rb * ROWS_B < R;

  bf16x8 kf[2][DS];
  uint4 vr[VROUNDS][2];             // raw V rows: 8 channels of one token per register quad

  // step -> (segment, first token, tokens in the segment)
  auto locate = [&](int st, const __bf16*& kp, const __bf16*& vp, long long& stride, int& tok0, int& len, bool& tree) {
    if (st < n0) { kp = k0; vp = v0; stride = a.token_stride; tok0 = st * STEP; len = Ls; tree = false; }
    else if (st < n0 + n1) { kp = k1; vp = v1; stride = a.token_stride; tok0 = (st - n0) * STEP; len = Lo; tree = false; }
    else { kp = k2; vp = v2; stride = stride2; tok0 = (st - n0 - n1) * STEP; len = n_b; tree = true; }
  };
  auto load_k = [&](int st) {
    const __bf16 *kp, *vp; long long stride; int tok0, len; bool tree;
    locate(st, kp, vp, stride, tok0, len, tree);
#pragma unroll
    for (int tt = 0; tt < 2; ++tt) {
      const int tok = min(tok0 + 16 * tt + col, len - 1);
      const __bf16* p = kp + (long long)tok * stride + 8 * qd;
#pragma unroll
      for (int j = 0; j < DS; ++j) kf[tt][j] = load_global_bf16x8(p + 32 * j);
    }
  };
  auto load_v = [&](int st) {
    const __bf16 *kp, *vp; long long stride; int tok0, len; bool tree;
    locate(st, kp, vp, stride, tok0, len, tree);
#pragma unroll
    for (int k = 0; k < VROUNDS; ++k) {
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const int tok = min(tok0 + 2 * TG * k + 2 * v_tg + h, len - 1);
        vr[k][h] = load_global_16(vp + (long long)tok * stride + 8 * v_dl);
      }
    }
  };

  int st = st_begin + tw;
  const bool active = block_live && st < st_end;
  if (active) { load_k(st); load_v(st); }
  // ---- topology of the tree (every wave for itself, while the first K/V loads travel): lane j = node j
  {
    uint64_t my_anc = 0;
    const int tb = dsbd_tree_walk(tr, lane, p_mine, a.max_depth, nullptr, reporter ? a.anc_out : nullptr, &my_anc);
    if (reporter && tb) atomicOr(a.fault, tb);
#pragma unroll
    for (int rt = 0; rt < NRT; ++rt) {
      const int r = row0 + rt * 16 + col;
      const int node = r < R ? r / a.group : 0;
      const unsigned lo = __shfl((unsigned)my_anc, node), hi = __shfl((unsigned)(my_anc >> 32), node);
      anc[rt] = r < R ? ((uint64_t)hi << 32) | lo : 0ull;
    }
  }

  // One step = 32 tokens of this wave: V goes to LDS transposed (two tokens packed per 32-bit write),
  // the next step's V and K loads are issued as soon as their registers are free, S^T = K Q^T.
  int tok0 = 0, nvalid = 0, st_next = 0;
  bool is_tree = false;
  floatx4 s[NRT][2];
  auto step_front = [&]() {
    const __bf16 *kp_, *vp_; long long stride_; int seglen;
    locate(st, kp_, vp_, stride_, tok0, seglen, is_tree);
    nvalid = min(STEP, seglen - tok0);
    st_next = st + TW;
    wave_lds_fence();
#pragma unroll
    for (int k = 0; k < VROUNDS; ++k) {
      const int tokp = 2 * TG * k + 2 * v_tg;          // even token index within the step
      const uint32_t ta[4] = {vr[k][0].x, vr[k][0].y, vr[k][0].z, vr[k][0].w};   // token tokp, channels 2c, 2c+1
      const uint32_t tb[4] = {vr[k][1].x, vr[k][1].y, vr[k][1].z, vr[k][1].w};   // token tokp + 1
#pragma unroll
      for (int c2 = 0; c2 < 4; ++c2) {
        // (token, token+1) pairs of channel 2c (low halves) and 2c+1 (high halves)
        const uint32_t lo = __builtin_amdgcn_perm(tb[c2], ta[c2], 0x05040100u);
        const uint32_t hi = __builtin_amdgcn_perm(tb[c2], ta[c2], 0x07060302u);
        *reinterpret_cast<uint32_t*>(&vt[(8 * v_dl + 2 * c2) * VT_PITCH + tokp]) = lo;
        *reinterpret_cast<uint32_t*>(&vt[(8 * v_dl + 2 * c2 + 1) * VT_PITCH + tokp]) = hi;
      }
    }
    wave_lds_fence();
    if (st_next < st_end) load_v(st_next);
#pragma unroll
    for (int rt = 0; rt < NRT; ++rt)
#pragma unroll
      for (int tt = 0; tt < 2; ++tt) {
        floatx4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int j = 0; j < DS; ++j) acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[tt][j], qf[rt][j], acc, 0, 0, 0);
        s[rt][tt] = acc;
      }
    if (st_next < st_end) load_k(st_next);
  };
  // O^T += V^T P^T
  auto step_pv = [&](const bf16x8 (&pf)[NRT]) {
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) {
      union { uint2 u[2]; bf16x8 v; } vf;
      const __bf16* rowp = &vt[(16 * dt + col) * VT_PITCH];
      vf.u[0] = *reinterpret_cast<const uint2*>(rowp + 4 * qd);
      vf.u[1] = *reinterpret_cast<const uint2*>(rowp + 16 + 4 * qd);
#pragma unroll
      for (int rt = 0; rt < NRT; ++rt) o[rt][dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf.v, pf[rt], o[rt][dt], 0, 0, 0);
    }
  };

  // Softmax numerators are taken against a per-row reference m_run that is NOT the exact running
  // maximum: it is set by the first step with a valid score for the row and raised only when a score
  // exceeds it by more than 2^REF_SLACK.  fp32 (and bf16, for P) have the exponent range for numerators
  // up to 2^REF_SLACK, and the final division by the row sum removes the reference.  So the hot loop
  // below is "exp2(s - m_run), accumulate": no rescaling of the output accumulators (which live in
  // accumulation registers that vector ALU instructions cannot touch), no cross-lane traffic.  Steps
  // that need a mask (tree rows, ragged tail) or a higher reference leave the hot loop and take the
  // general path once.
  while (active && st < st_end) {
    bool general = false;
    while (st < st_end) {                      // ---- hot loop
      step_front();
      if (is_tree || nvalid < STEP) { general = true; break; }
      bool raise = false;
#pragma unroll
      for (int rt = 0; rt < NRT; ++rt) {
        float mx = fmaxf(fmaxf(s[rt][0][0], s[rt][0][1]), fmaxf(s[rt][0][2], s[rt][0][3]));
        mx = fmaxf(mx, fmaxf(fmaxf(s[rt][1][0], s[rt][1][1]), fmaxf(s[rt][1][2], s[rt][1][3])));
        raise = raise || (mx * a.scale_log2 > m_run[rt] + REF_SLACK);
      }
      if (__builtin_amdgcn_ballot_w64(raise) != 0ull) { general = true; break; }
      bf16x8 pf[NRT];
#pragma unroll
      for (int rt = 0; rt < NRT; ++rt) {
        const float nm = -m_run[rt];
        float psum = 0.f;
#pragma unroll
        for (int tt = 0; tt < 2; ++tt)
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const float p = __builtin_amdgcn_exp2f(fmaf(s[rt][tt][i], a.scale_log2, nm));
            psum += p;
            pf[rt][4 * tt + i] = (__bf16)p;
          }
        l_run[rt] += psum;
      }
      step_pv(pf);
      st = st_next;
    }
    if (!general) break;

    // ---- general step: masks, reference raise with rescaling
    const bool need_mask = is_tree || nvalid < STEP;
    bf16x8 pf[NRT];
#pragma unroll
    for (int rt = 0; rt < NRT; ++rt) {
      float sv[8];
#pragma unroll
      for (int tt = 0; tt < 2; ++tt)
#pragma unroll
        for (int i = 0; i < 4; ++i) sv[4 * tt + i] = s[rt][tt][i] * a.scale_log2;
      unsigned okbits = 0xffu;
      if (need_mask) {
        okbits = 0;
#pragma unroll
        for (int tt = 0; tt < 2; ++tt)
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const int t = 16 * tt + 4 * qd + i;          // token within the step
            bool valid = t < nvalid;
            if (is_tree) valid = valid && ((anc[rt] >> (tok0 + t)) & 1ull);
            if (valid) okbits |= 1u << (4 * tt + i); else sv[4 * tt + i] = NEG_BIG;
          }
      }
      float mx = fmaxf(fmaxf(fmaxf(sv[0], sv[1]), fmaxf(sv[2], sv[3])), fmaxf(fmaxf(sv[4], sv[5]), fmaxf(sv[6], sv[7])));
      mx = fmaxf(mx, __shfl_xor(mx, 16));
      mx = fmaxf(mx, __shfl_xor(mx, 32));                  // same value in the 4 lane groups of a row
      const float m_new = (mx > m_run[rt] + REF_SLACK) ? mx : m_run[rt];
      const float alpha = __builtin_amdgcn_exp2f(m_run[rt] - m_new);
      l_run[rt] *= alpha;
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) o[rt][dt] *= alpha;
      m_run[rt] = m_new;
      float psum = 0.f;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float p = ((okbits >> e) & 1u) ? __builtin_amdgcn_exp2f(sv[e] - m_new) : 0.f;
        psum += p;
        pf[rt][e] = (__bf16)p;
      }
      l_run[rt] += psum;
    }
    step_pv(pf);
    st = st_next;
  }

  // ---- finish the row sums (each lane group summed its own tokens)
#pragma unroll
  for (int rt = 0; rt < NRT; ++rt) {
    l_run[rt] += __shfl_xor(l_run[rt], 16);
    l_run[rt] += __shfl_xor(l_run[rt], 32);
  }

  // ---- merge the token groups of the workgroup through LDS
  if (TW > 1) {
    if (tw > 0) {
      const int slot = (tw - 1) * RW + rw;
#pragma unroll
      for (int rt = 0; rt < NRT; ++rt) {
        const int rloc = rt * 16 + col;
        if (qd == 0) { comb_ml[slot][rloc][0] = m_run[rt]; comb_ml[slot][rloc][1] = l_run[rt]; }
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
          *reinterpret_cast<floatx4*>(&comb_o[slot][rloc][16 * dt + 4 * qd]) = o[rt][dt];
      }
    }
    __syncthreads();
    if (tw == 0) {
      for (int t2 = 1; t2 < TW; ++t2) {
        const int slot = (t2 - 1) * RW + rw;
#pragma unroll
        for (int rt = 0; rt < NRT; ++rt) {
          const int rloc = rt * 16 + col;
          const float m2 = comb_ml[slot][rloc][0], l2 = comb_ml[slot][rloc][1];
          const float m_new = fmaxf(m_run[rt], m2);
          const float a1 = exp2f(m_run[rt] - m_new), a2 = exp2f(m2 - m_new);
          l_run[rt] = l_run[rt] * a1 + l2 * a2;
          m_run[rt] = m_new;
#pragma unroll
          for (int dt = 0; dt < DT; ++dt) {
            const floatx4 o2 = *reinterpret_cast<const floatx4*>(&comb_o[slot][rloc][16 * dt + 4 * qd]);
            o[rt][dt] = o[rt][dt] * a1 + o2 * a2;
          }
        }
      }
    }
  }

  // ---- partial results of this split
  if (tw == 0) {
#pragma unroll
    for (int rt = 0; rt < NRT; ++rt) {
      const int r = row0 + rt * 16 + col;
      if (r < R) {
        const int node = r / a.group;
        const int head = g * a.group + r % a.group;
        const long long grow = (long long)(base + node) * a.Hq + head;
        const long long prow = (long long)split * n_rows_total + grow;
        if (qd == 0) { a.part_ml[prow * 2] = m_run[rt]; a.part_ml[prow * 2 + 1] = l_run[rt]; }
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
          *reinterpret_cast<floatx4*>(&a.part_o[prow * D + 16 * dt + 4 * qd]) = o[rt][dt];
      }
    }
  }
}

// ------------------------------------------------------------------------------------------------
// Variant for many query rows per K/V stream (large trees and/or grouped-query attention): the RW
// waves of a workgroup each keep 32 query rows (two 16-row tiles) and ALL consume the same 64-token
// K/V tile, which is staged once through LDS, both row-major with padded rows: K is read back as MFMA A operands
// with 16-byte reads, V through the transposing LDS read of gfx950 (ds_read_b64_tr_b16), which hands a lane four
// tokens of one channel.  Tiles are double-buffered: while tile t
// is consumed from one buffer, tile t+1 sits in registers on its way to the other buffer and tile t+2
// is in flight from HBM; one workgroup barrier per tile.  Two workgroups fit a CU (<= 256 registers,
// < 80 KiB LDS), so one can compute while the other waits on memory.
template <int D, int RW, int NRT>
__global__ __launch_bounds__(64 * RW) __attribute__((amdgpu_waves_per_eu(NRT == 1 ? 4 : 2, NRT == 1 ? 4 : 2)))
void forest_attention_shared_kernel(AttnArgs a) {
  constexpr int NT = 64 * RW;
  constexpr int TILE = 64;
  constexpr int DS = D / 32, DT = D / 16;
  constexpr int CG = D / 8;                 // 16-byte channel groups per row
  constexpr int KP = D + 8;                 // K row pitch in elements (16 bytes of padding)
  constexpr int KL = TILE * CG / NT;        // K 16-byte loads per thread and tile
  constexpr int ROWS_W = 16 * NRT, ROWS_B = ROWS_W * RW;

  constexpr int OP = D + 4;                 // row pitch (floats) of the output staging tile
  constexpr int TILE_BYTES = 2 * (TILE * KP + TILE * KP) * 2;
  constexpr int OUT_BYTES = ROWS_B * OP * 4;
  __shared__ __attribute__((aligned(16))) char smem[TILE_BYTES > OUT_BYTES ? TILE_BYTES : OUT_BYTES];
  __bf16 (*k_lds)[TILE * KP] = reinterpret_cast<__bf16 (*)[TILE * KP]>(smem);
  __bf16 (*v_lds)[TILE * KP] = reinterpret_cast<__bf16 (*)[TILE * KP]>(smem + 2 * TILE * KP * 2);
  float* o_stage = reinterpret_cast<float*>(smem);   // reused after the last tile

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int col = lane & 15, qd = lane >> 4;

  int bid = blockIdx.x;
  const int split = bid % a.nsplit; bid /= a.nsplit;
  const int rb = bid % a.n_rowblocks; bid /= a.n_rowblocks;
  const int g = bid % a.Hkv;
  const int b = bid / a.Hkv;

  const dsbd_tree_range tr = dsbd_tree_range_of(b, a.n_nodes, a.tree_off, a.max_tree_nodes);
  const bool reporter = split == 0 && rb == 0 && g == 0 && wave == 0;   // one wave per tree speaks for it
  if (!tr.valid) {
    if (reporter && lane == 0) atomicOr(a.fault, tr.bad);
    return;
  }
  const int base = tr.base;
  const int n_b = min(tr.n_all, DSBD_MAX_TREE_NODES);
  const int p_mine = dsbd_tree_parent_of(tr, lane, a.parent);   // used once the first loads are on their way
  const int R = n_b * a.group;
  if (rb * ROWS_B >= R) return;             // uniform over the workgroup
  const int row0 = rb * ROWS_B + wave * ROWS_W;
  const int n_rows_total = a.n_nodes * a.Hq;

  int Ls = (a.shared_len && a.k_shared_ptr) ? a.shared_len[b] : 0;
  int Lo = a.len[b];
  Ls = max(Ls, 0); Lo = max(Lo, 0);
  int bad = 0;
  if ((long long)Ls + Lo > a.max_len) { bad |= DSBD_FAULT_BOUNDS; Ls = min(Ls, a.max_len); Lo = min(Lo, a.max_len - Ls); }
  const long long hoff = (long long)g * a.head_stride;
  const __bf16* k0 = Ls ? (const __bf16*)a.k_shared_ptr[b] : nullptr;
  const __bf16* v0 = Ls ? (const __bf16*)a.v_shared_ptr[b] : nullptr;
  const __bf16* k1 = Lo ? (const __bf16*)a.k_ptr[b] : nullptr;
  const __bf16* v1 = Lo ? (const __bf16*)a.v_ptr[b] : nullptr;
  if (Ls && (!k0 || !v0 || (((uintptr_t)k0 | (uintptr_t)v0) & 15))) { bad |= DSBD_FAULT_BOUNDS; Ls = 0; }
  if (Lo && (!k1 || !v1 || (((uintptr_t)k1 | (uintptr_t)v1) & 15))) { bad |= DSBD_FAULT_BOUNDS; Lo = 0; }
  if (bad && tid == 0) atomicOr(a.fault, bad);
  k0 += hoff; v0 += hoff; k1 += hoff; v1 += hoff;
  const __bf16* k2 = a.k_tree + ((long long)base * a.Hkv + g) * D;
  const __bf16* v2 = a.v_tree + ((long long)base * a.Hkv + g) * D;
  const long long stride2 = (long long)a.Hkv * D;
  const int n0 = (Ls + TILE - 1) / TILE, n1 = (Lo + TILE - 1) / TILE, n2 = (n_b + TILE - 1) / TILE;
  const int total_tiles = n0 + n1 + n2;
  // balanced partition: the first (total % nsplit) splits take one tile more than the others (with ceil-sized
  // splits the last one came out 7 tiles short on the benchmark shape and one XCD idled for a third of the kernel)
  const int t_begin = split * (total_tiles / a.nsplit) + min(split, total_tiles % a.nsplit);
  const int t_end = t_begin + total_tiles / a.nsplit + (split < total_tiles % a.nsplit ? 1 : 0);

  // resident query fragments and ancestor bitmaps
  bf16x8 qf[NRT][DS];
  uint64_t anc[NRT];
#pragma unroll
  for (int rt = 0; rt < NRT; ++rt) {
    const int r = row0 + rt * 16 + col;
    const bool live = r < R;
    const int node = live ? r / a.group : 0;
    const int head = g * a.group + (live ? r % a.group : 0);
    anc[rt] = 0ull;
    const __bf16* qp = a.q + ((long long)(base + node) * a.Hq + head) * D + 8 * qd;
#pragma unroll
    for (int j = 0; j < DS; ++j) {
      if (live) {
        qf[rt][j] = load_global_bf16x8(qp + 32 * j);
      } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) qf[rt][j][e] = (__bf16)0.0f;
      }
    }
  }
  floatx4 o[NRT][DT];
  float m_run[NRT], l_run[NRT];
#pragma unroll
  for (int rt = 0; rt < NRT; ++rt) {
    m_run[rt] = NEG_BIG; l_run[rt] = 0.f;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) o[rt][dt] = floatx4{0.f, 0.f, 0.f, 0.f};
  }

  auto locate = [&](int ti, const __bf16*& kp, const __bf16*& vp, long long& stride, int& tok0, int& len, bool& tree) {
    if (ti < n0) { kp = k0; vp = v0; stride = a.token_stride; tok0 = ti * TILE; len = Ls; tree = false; }
    else if (ti < n0 + n1) { kp = k1; vp = v1; stride = a.token_stride; tok0 = (ti - n0) * TILE; len = Lo; tree = false; }
    else { kp = k2; vp = v2; stride = stride2; tok0 = (ti - n0 - n1) * TILE; len = n_b; tree = true; }
  };

  // optional timeline of workgroup 0 / thread 0 (build with -DDSBD_ATTN_TIMELINE, run with DSBD_ATTN_TRACE
  // set): stamps are kept in LDS and copied out at the end, so that taking them adds no global-memory
  // traffic to the waits being measured
#ifdef DSBD_ATTN_TIMELINE
  const long long wg_start = wall_clock64();
  __shared__ long long trace_lds[2 * 120];
  int trace_n = 0;
  const bool tracing = a.trace != nullptr && blockIdx.x == 0 && tid == 0;
  auto stamp = [&](int label) {
    if (tracing && trace_n < 120) { trace_lds[2 * trace_n] = label; trace_lds[2 * trace_n + 1] = wall_clock64(); ++trace_n; }
  };
#else
  auto stamp = [&](int) {};
#endif
  uint4 kreg[KL];
  uint4 vreg[KL];
  auto load_tile = [&](int ti) {
    const __bf16 *kp, *vp; long long stride; int tok0, len; bool tree;
    locate(ti, kp, vp, stride, tok0, len, tree);
#pragma unroll
    for (int r = 0; r < KL; ++r) {            // CG consecutive lanes read one whole token row of K and of V
      const int c = r * NT + tid;
      const int tok = min(tok0 + c / CG, len - 1);
      const long long off = (long long)tok * stride + (c % CG) * 8;
      kreg[r] = load_global_16_nt(kp + off);
      vreg[r] = load_global_16_nt(vp + off);
    }
  };
  auto store_tile = [&](int buf) {
    __bf16* kl = k_lds[buf];
    __bf16* vl = v_lds[buf];
#pragma unroll
    for (int r = 0; r < KL; ++r) {
      const int c = r * NT + tid;
      *reinterpret_cast<uint4*>(&kl[(c / CG) * KP + (c % CG) * 8]) = kreg[r];
      *reinterpret_cast<uint4*>(&vl[(c / CG) * KP + (c % CG) * 8]) = vreg[r];
    }
  };

  int ti = t_begin;
  if (ti < t_end) load_tile(ti);
  // ---- topology of the tree (every wave for itself, while the first K/V loads travel): lane j = node j
  {
    uint64_t my_anc = 0;
    const int tb = dsbd_tree_walk(tr, lane, p_mine, a.max_depth, nullptr, reporter ? a.anc_out : nullptr, &my_anc);
    if (reporter && tb) atomicOr(a.fault, tb);
#pragma unroll
    for (int rt = 0; rt < NRT; ++rt) {
      const int r = row0 + rt * 16 + col;
      const int node = r < R ? r / a.group : 0;
      const unsigned lo = __shfl((unsigned)my_anc, node), hi = __shfl((unsigned)(my_anc >> 32), node);
      anc[rt] = r < R ? ((uint64_t)hi << 32) | lo : 0ull;
    }
  }
  // Everything requested so far (query fragments, ancestor bitmaps, the first tile) is needed now anyway.
  // Waiting for it explicitly, at a point that dominates the loop, keeps the compiler from re-waiting for
  // the query loads at the loop header with a vmcnt(0) that would also drain the prefetched tile.
  __builtin_amdgcn_s_waitcnt(0x0F70);      // vmcnt(0), other counters untouched
  if (ti < t_end) store_tile(0);
  lds_barrier();
  if (ti + 1 < t_end) load_tile(ti + 1);
  int buf = 0;

  while (ti < t_end) {
    const __bf16 *kp_, *vp_; long long stride_; int tok0, seglen; bool is_tree;
    locate(ti, kp_, vp_, stride_, tok0, seglen, is_tree);
    const int nvalid = min(TILE, seglen - tok0);
    const __bf16* kl = k_lds[buf];
    const __bf16* vl = v_lds[buf];

    stamp(1);
    // The tile is consumed in two 32-token halves (scores -> numerators -> O^T update per half), which keeps
    // only 16 score and 8 numerator registers live next to the accumulators, so that the registers holding
    // the NEXT tile's in-flight loads are never touched (a spill or reuse of them would force a wait for
    // all outstanding K/V loads before the arithmetic, exposing the memory latency every tile).
    const bool need_mask = is_tree || nvalid < TILE;
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
      // ---- S^T = K Q^T: 2 token tiles x NRT row tiles
      floatx4 s[NRT][2];
#pragma unroll
      for (int t2 = 0; t2 < 2; ++t2) {
#pragma unroll
        for (int rt = 0; rt < NRT; ++rt) s[rt][t2] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int j = 0; j < DS; ++j) {
          const bf16x8 kfrag = *reinterpret_cast<const bf16x8*>(&kl[(32 * ks + 16 * t2 + col) * KP + 32 * j + 8 * qd]);
#pragma unroll
          for (int rt = 0; rt < NRT; ++rt)
            s[rt][t2] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kfrag, qf[rt][j], s[rt][t2], 0, 0, 0);
        }
      }
      // ---- softmax numerators against the per-row reference (see forest_attention_kernel)
      bf16x8 pf[NRT];
      bool raise = false;
#pragma unroll
      for (int rt = 0; rt < NRT; ++rt) {
        float mx = fmaxf(fmaxf(s[rt][0][0], s[rt][0][1]), fmaxf(s[rt][0][2], s[rt][0][3]));
        mx = fmaxf(mx, fmaxf(fmaxf(s[rt][1][0], s[rt][1][1]), fmaxf(s[rt][1][2], s[rt][1][3])));
        raise = raise || (mx * a.scale_log2 > m_run[rt] + REF_SLACK);
      }
      if (!need_mask && __builtin_amdgcn_ballot_w64(raise) == 0ull) {
#pragma unroll
        for (int rt = 0; rt < NRT; ++rt) {
          const float nm = -m_run[rt];
          float psum = 0.f;
#pragma unroll
          for (int t2 = 0; t2 < 2; ++t2)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
              const float p = __builtin_amdgcn_exp2f(fmaf(s[rt][t2][i], a.scale_log2, nm));
              psum += p;
              pf[rt][4 * t2 + i] = (__bf16)p;
            }
          l_run[rt] += psum;
        }
      } else {
#pragma unroll
        for (int rt = 0; rt < NRT; ++rt) {
          float sv[8];
          unsigned okbits = 0;
#pragma unroll
          for (int t2 = 0; t2 < 2; ++t2)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
              const int t = 32 * ks + 16 * t2 + 4 * qd + i;          // token within the tile
              bool valid = t < nvalid;
              if (is_tree) valid = valid && ((anc[rt] >> (tok0 + t)) & 1ull);
              if (valid) okbits |= 1u << (4 * t2 + i);
              sv[4 * t2 + i] = valid ? s[rt][t2][i] * a.scale_log2 : NEG_BIG;
            }
          float mx = sv[0];
#pragma unroll
          for (int e = 1; e < 8; ++e) mx = fmaxf(mx, sv[e]);
          mx = fmaxf(mx, __shfl_xor(mx, 16));
          mx = fmaxf(mx, __shfl_xor(mx, 32));
          const float m_new = (mx > m_run[rt] + REF_SLACK) ? mx : m_run[rt];
          const float alpha = __builtin_amdgcn_exp2f(m_run[rt] - m_new);
          l_run[rt] *= alpha;
#pragma unroll
          for (int dt = 0; dt < DT; ++dt) o[rt][dt] *= alpha;
          m_run[rt] = m_new;
          float psum = 0.f;
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            const float p = ((okbits >> e) & 1u) ? __builtin_amdgcn_exp2f(sv[e] - m_new) : 0.f;
            psum += p;
            pf[rt][e] = (__bf16)p;
          }
          l_run[rt] += psum;
        }
      }
      // ---- O^T += V^T P^T for this half
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) {
        // A operand = V^T: lane (channel 16dt + col, qd) needs tokens 4qd .. 4qd+3 of both 16-token blocks of the
        // half, the order the numerators have in pf.  A transposing read returns, to lane i of a group of 16, the
        // element i % 4 of the four lanes i / 4, 4 + i / 4, ...: so lane i points at token 4qd + i / 4, channels
        // 16dt + 4 (i % 4) .. + 3, and receives channel 16dt + i of tokens 4qd .. 4qd+3.
        union { v4i16 h[2]; bf16x8 v; } vf;
        const __bf16* rowp = &vl[(32 * ks + 4 * qd + (col >> 2)) * KP + 16 * dt + 4 * (col & 3)];
        vf.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4i16*)(rowp));
        vf.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4i16*)(rowp + 16 * KP));
#pragma unroll
        for (int rt = 0; rt < NRT; ++rt)
          o[rt][dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf.v, pf[rt], o[rt][dt], 0, 0, 0);
      }
    }

    // ---- advance the pipeline: tile ti+1 (in registers) goes to the other LDS buffer, whose readers all
    // passed the barrier that ended the previous iteration; then tile ti+2 is requested and travels during
    // the next tile's arithmetic.  (Requesting it before this iteration's arithmetic measured slower.)
    stamp(4);
    if (ti + 1 < t_end) store_tile(buf ^ 1);
    stamp(5);
    if (ti + 2 < t_end) load_tile(ti + 2);
    stamp(6);
    lds_barrier();
    buf ^= 1;
    ++ti;
  }

  // ---- partial results of this split: (m, l) per row, and O^T turned back into rows through LDS so
  // that every row leaves as one contiguous 4*D-byte write instead of 16-byte pieces
#pragma unroll
  for (int rt = 0; rt < NRT; ++rt) {
    l_run[rt] += __shfl_xor(l_run[rt], 16);
    l_run[rt] += __shfl_xor(l_run[rt], 32);
    const int rl = wave * ROWS_W + rt * 16 + col;          // row within the block
    const int r = rb * ROWS_B + rl;
    if (r < R && qd == 0) {
      const int node = r / a.group;
      const int head = g * a.group + r % a.group;
      const long long prow = (long long)split * n_rows_total + (long long)(base + node) * a.Hq + head;
      a.part_ml[prow * 2] = m_run[rt];
      a.part_ml[prow * 2 + 1] = l_run[rt];
    }
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
      *reinterpret_cast<floatx4*>(&o_stage[rl * OP + 16 * dt + 4 * qd]) = o[rt][dt];
  }
  __syncthreads();
  constexpr int LPR_O = D / 4;              // lanes per output row (16 bytes each)
  for (int c = tid; c < ROWS_B * LPR_O; c += NT) {
    const int rl = c / LPR_O, part = c % LPR_O;
    const int r = rb * ROWS_B + rl;
    if (r < R) {
      const int node = r / a.group;
      const int head = g * a.group + r % a.group;
      const long long prow = (long long)split * n_rows_total + (long long)(base + node) * a.Hq + head;
      *reinterpret_cast<floatx4*>(&a.part_o[prow * D + 4 * part]) = *reinterpret_cast<const floatx4*>(&o_stage[rl * OP + 4 * part]);
    }
  }
#ifdef DSBD_ATTN_TIMELINE
  if (a.trace != nullptr && tid == 0 && blockIdx.x < 1024) {     // start / end of every workgroup
    a.trace[1024 + 2 * blockIdx.x] = wg_start;
    a.trace[1024 + 2 * blockIdx.x + 1] = wall_clock64();
  }
  if (tracing) {
    a.trace[0] = trace_n;
    for (int i = 0; i < 2 * trace_n; ++i) a.trace[2 + i] = trace_lds[i];
  }
#endif
}

// ------------------------------------------------------------------------------------------------
// The shared-tile kernel with the K/V tiles loaded straight into the LDS (global_load_lds_dwordx4: a wave's 64
// lanes fill 1 KiB of consecutive LDS, no staging registers, no LDS stores).  Rows cannot be padded that way, so
// bank conflicts are avoided by a swizzle instead: the 16-byte piece p of token t sits at position p ^ f(t) of the
// token's 256-byte row, f(t) = 2 (t & 3) + ((t >> 2) & 1), which spreads both the K operand reads (16 consecutive
// tokens, one piece) and the transposing V reads (4 consecutive tokens, two pieces) over all banks.  The two
// tile buffers are four separate LDS arrays and the loop is written out for both, so that the compiler can tell
// a read of one buffer from the load in flight into the other (it waits for every outstanding LDS-bound load
// before an LDS read that may alias it).  D = 128, four waves of 32 rows.  Measured against the kernel above on the
// benchmark shape: 60.5 us against 62.5 (fewer registers, no LDS stores, whole tiles addressed without per-lane
// arithmetic); a variant with 32-token tiles and three waves per SIMD (168 registers, 11 of them spilled) took 68 us.
#ifndef DSBD_DMA_AUX
#define DSBD_DMA_AUX 2        // cache policy of the tile loads: non-temporal, as in the shared-tile kernel
#endif
typedef __attribute__((address_space(3))) void lds_void_t;
typedef __attribute__((address_space(1))) const void glb_cvoid_t;
template <int TILE, int WPE>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(WPE, WPE)))
void forest_attention_dma_kernel(AttnArgs a) {
  constexpr int D = 128, RW = 4, NRT = 2;
  constexpr int DS = D / 32, DT = D / 16;
  constexpr int SLOTS = TILE * 16;          // 16-byte slots of a K or V tile
  constexpr int ROWS_W = 16 * NRT, ROWS_B = ROWS_W * RW;
  __shared__ __attribute__((aligned(16))) uint4 kA[SLOTS];
  __shared__ __attribute__((aligned(16))) uint4 kB[SLOTS];
  __shared__ __attribute__((aligned(16))) uint4 vA[SLOTS];
  __shared__ __attribute__((aligned(16))) uint4 vB[SLOTS];

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int col = lane & 15, qd = lane >> 4;

  int bid = blockIdx.x;
  const int split = bid % a.nsplit; bid /= a.nsplit;
  const int rb = bid % a.n_rowblocks; bid /= a.n_rowblocks;
  const int g = bid % a.Hkv;
  const int b = bid / a.Hkv;

  const dsbd_tree_range tr = dsbd_tree_range_of(b, a.n_nodes, a.tree_off, a.max_tree_nodes);
  const bool reporter = split == 0 && rb == 0 && g == 0 && wave == 0;
  if (!tr.valid) {
    if (reporter && lane == 0) atomicOr(a.fault, tr.bad);
    return;
  }
  const int base = tr.base;
  const int n_b = min(tr.n_all, DSBD_MAX_TREE_NODES);
  const int p_mine = dsbd_tree_parent_of(tr, lane, a.parent);
  const int R = n_b * a.group;
  if (rb * ROWS_B >= R) return;
  const int row0 = rb * ROWS_B + wave * ROWS_W;
  const int n_rows_total = a.n_nodes * a.Hq;

  int Ls = (a.shared_len && a.k_shared_ptr) ? a.shared_len[b] : 0;
  int Lo = a.len[b];
  Ls = max(Ls, 0); Lo = max(Lo, 0);
  int bad = 0;
  if ((long long)Ls + Lo > a.max_len) { bad |= DSBD_FAULT_BOUNDS; Ls = min(Ls, a.max_len); Lo = min(Lo, a.max_len - Ls); }
  const long long hoff = (long long)g * a.head_stride;
  const __bf16* k0 = Ls ? (const __bf16*)a.k_shared_ptr[b] : nullptr;
  const __bf16* v0 = Ls ? (const __bf16*)a.v_shared_ptr[b] : nullptr;
  const __bf16* k1 = Lo ? (const __bf16*)a.k_ptr[b] : nullptr;
  const __bf16* v1 = Lo ? (const __bf16*)a.v_ptr[b] : nullptr;
  if (Ls && (!k0 || !v0 || (((uintptr_t)k0 | (uintptr_t)v0) & 15))) { bad |= DSBD_FAULT_BOUNDS; Ls = 0; }
  if (Lo && (!k1 || !v1 || (((uintptr_t)k1 | (uintptr_t)v1) & 15))) { bad |= DSBD_FAULT_BOUNDS; Lo = 0; }
  if (bad && tid == 0) atomicOr(a.fault, bad);
  k0 += hoff; v0 += hoff; k1 += hoff; v1 += hoff;
  const __bf16* k2 = a.k_tree + ((long long)base * a.Hkv + g) * D;
  const __bf16* v2 = a.v_tree + ((long long)base * a.Hkv + g) * D;
  const long long stride2 = (long long)a.Hkv * D;
  const int n0 = (Ls + TILE - 1) / TILE, n1 = (Lo + TILE - 1) / TILE, n2 = (n_b + TILE - 1) / TILE;
  const int total_tiles = n0 + n1 + n2;
  const int t_begin = split * (total_tiles / a.nsplit) + min(split, total_tiles % a.nsplit);
  const int t_end = t_begin + total_tiles / a.nsplit + (split < total_tiles % a.nsplit ? 1 : 0);

  bf16x8 qf[NRT][DS];
  uint64_t anc[NRT];
#pragma unroll
  for (int rt = 0; rt < NRT; ++rt) {
    const int r = row0 + rt * 16 + col;
    const bool live = r < R;
    const int node = live ? r / a.group : 0;
    const int head = g * a.group + (live ? r % a.group : 0);
    anc[rt] = 0ull;
    const __bf16* qp = a.q + ((long long)(base + node) * a.Hq + head) * D + 8 * qd;
#pragma unroll
    for (int j = 0; j < DS; ++j) {
      if (live) {
        qf[rt][j] = load_global_bf16x8(qp + 32 * j);
      } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) qf[rt][j][e] = (__bf16)0.0f;
      }
    }
  }
  floatx4 o[NRT][DT];
  float m_run[NRT], l_run[NRT];
#pragma unroll
  for (int rt = 0; rt < NRT; ++rt) {
    m_run[rt] = NEG_BIG; l_run[rt] = 0.f;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) o[rt][dt] = floatx4{0.f, 0.f, 0.f, 0.f};
  }

  auto locate = [&](int ti, const __bf16*& kp, const __bf16*& vp, long long& stride, int& tok0, int& len, bool& tree) {
    if (ti < n0) { kp = k0; vp = v0; stride = a.token_stride; tok0 = ti * TILE; len = Ls; tree = false; }
    else if (ti < n0 + n1) { kp = k1; vp = v1; stride = a.token_stride; tok0 = (ti - n0) * TILE; len = Lo; tree = false; }
    else { kp = k2; vp = v2; stride = stride2; tok0 = (ti - n0 - n1) * TILE; len = n_b; tree = true; }
  };
  auto swz = [](int t) { return ((t & 3) << 1) | ((t >> 2) & 1); };
  // tile ti -> the LDS arrays Kb / Vb: instruction r of wave w fills slots (4r + w) * 64 .. + 63, i.e. lane L fills
  // position L % 16 of token 4 (4r + w) + L / 16 and therefore fetches piece (L % 16) ^ f(token)
  const int ld_piece = (lane & 15) ^ swz((lane >> 4) + 4 * wave);          // (4 (4r + w)) & 7 = 4 (w & 1): f's last bit
  // A whole tile (no ragged end) needs no per-lane arithmetic at all: the lane's byte offset inside the tile's
  // first 16 tokens is a constant of the segment, the tile and the 16-token step are uniform.
  const int ld_tok = 4 * wave + (lane >> 4);
  auto issue = [&](int ti, auto& Kb, auto& Vb) {
    const __bf16 *kp, *vp; long long stride; int tok0, len; bool tree;
    locate(ti, kp, vp, stride, tok0, len, tree);
    if (tok0 + TILE <= len) {
      const char* const kb = reinterpret_cast<const char*>(kp + (long long)tok0 * stride);
      const char* const vb = reinterpret_cast<const char*>(vp + (long long)tok0 * stride);
      const unsigned int lo = (unsigned int)ld_tok * (unsigned int)(stride * 2) + (unsigned int)(ld_piece * 16);
#pragma unroll
      for (int r = 0; r < TILE / 16; ++r) {
        const long long step = (long long)r * 16 * stride * 2;
        __builtin_amdgcn_global_load_lds((glb_cvoid_t*)(kb + step + lo), (lds_void_t*)&Kb[(4 * r + wave) * 64], 16, 0, DSBD_DMA_AUX);
        __builtin_amdgcn_global_load_lds((glb_cvoid_t*)(vb + step + lo), (lds_void_t*)&Vb[(4 * r + wave) * 64], 16, 0, DSBD_DMA_AUX);
      }
      return;
    }
#pragma unroll
    for (int r = 0; r < TILE / 16; ++r) {
      const int t = 4 * (4 * r + wave) + (lane >> 4);
      const int tok = min(tok0 + t, len - 1);
      const long long off = (long long)tok * stride + ld_piece * 8;
      __builtin_amdgcn_global_load_lds((glb_cvoid_t*)(kp + off), (lds_void_t*)&Kb[(4 * r + wave) * 64], 16, 0, DSBD_DMA_AUX);
      __builtin_amdgcn_global_load_lds((glb_cvoid_t*)(vp + off), (lds_void_t*)&Vb[(4 * r + wave) * 64], 16, 0, DSBD_DMA_AUX);
    }
  };
  // byte offsets of this lane's operand reads inside a tile, without the token-block part (a multiple of 4 KiB)
  int k_off[DS];                             // K: token col, piece (4 j + qd) ^ f(col)
#pragma unroll
  for (int j = 0; j < DS; ++j) k_off[j] = col * 256 + (((4 * j + qd) ^ swz(col)) << 4);
  int v_off[DT];                             // V: token 4 qd + col / 4, piece (2 dt + (col & 3) / 2) ^ f, half col & 1
#pragma unroll
  for (int dt = 0; dt < DT; ++dt) {
    const int t = 4 * qd + (col >> 2);
    v_off[dt] = t * 256 + (((2 * dt + ((col & 3) >> 1)) ^ swz(t)) << 4) + ((col & 1) << 3);
  }

  auto compute = [&](int ti, auto& Kb, auto& Vb) {
    const __bf16 *kp_, *vp_; long long stride_; int tok0, seglen; bool is_tree;
    locate(ti, kp_, vp_, stride_, tok0, seglen, is_tree);
    const int nvalid = min(TILE, seglen - tok0);
    const char* const kl = reinterpret_cast<const char*>(&Kb[0]);
    const char* const vl = reinterpret_cast<const char*>(&Vb[0]);
    const bool need_mask = is_tree || nvalid < TILE;
#pragma unroll
    for (int ks = 0; ks < TILE / 32; ++ks) {
      floatx4 s[NRT][2];
#pragma unroll
      for (int t2 = 0; t2 < 2; ++t2) {
#pragma unroll
        for (int rt = 0; rt < NRT; ++rt) s[rt][t2] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int j = 0; j < DS; ++j) {
          const bf16x8 kfrag = *reinterpret_cast<const bf16x8*>(kl + (32 * ks + 16 * t2) * 256 + k_off[j]);
#pragma unroll
          for (int rt = 0; rt < NRT; ++rt)
            s[rt][t2] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kfrag, qf[rt][j], s[rt][t2], 0, 0, 0);
        }
      }
      bf16x8 pf[NRT];
      bool raise = false;
#pragma unroll
      for (int rt = 0; rt < NRT; ++rt) {
        float mx = fmaxf(fmaxf(s[rt][0][0], s[rt][0][1]), fmaxf(s[rt][0][2], s[rt][0][3]));
        mx = fmaxf(mx, fmaxf(fmaxf(s[rt][1][0], s[rt][1][1]), fmaxf(s[rt][1][2], s[rt][1][3])));
        raise = raise || (mx * a.scale_log2 > m_run[rt] + REF_SLACK);
      }
      if (!need_mask && __builtin_amdgcn_ballot_w64(raise) == 0ull) {
#pragma unroll
        for (int rt = 0; rt < NRT; ++rt) {
          const float nm = -m_run[rt];
          float psum = 0.f;
#pragma unroll
          for (int t2 = 0; t2 < 2; ++t2)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
              const float p = __builtin_amdgcn_exp2f(fmaf(s[rt][t2][i], a.scale_log2, nm));
              psum += p;
              pf[rt][4 * t2 + i] = (__bf16)p;
            }
          l_run[rt] += psum;
        }
      } else {
#pragma unroll
        for (int rt = 0; rt < NRT; ++rt) {
          float sv[8];
          unsigned okbits = 0;
#pragma unroll
          for (int t2 = 0; t2 < 2; ++t2)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
              const int t = 32 * ks + 16 * t2 + 4 * qd + i;
              bool valid = t < nvalid;
              if (is_tree) valid = valid && ((anc[rt] >> (tok0 + t)) & 1ull);
              if (valid) okbits |= 1u << (4 * t2 + i);
              sv[4 * t2 + i] = valid ? s[rt][t2][i] * a.scale_log2 : NEG_BIG;
            }
          float mx = sv[0];
#pragma unroll
          for (int e = 1; e < 8; ++e) mx = fmaxf(mx, sv[e]);
          mx = fmaxf(mx, __shfl_xor(mx, 16));
          mx = fmaxf(mx, __shfl_xor(mx, 32));
          const float m_new = (mx > m_run[rt] + REF_SLACK) ? mx : m_run[rt];
          const float alpha = __builtin_amdgcn_exp2f(m_run[rt] - m_new);
          l_run[rt] *= alpha;
#pragma unroll
          for (int dt = 0; dt < DT; ++dt) o[rt][dt] *= alpha;
          m_run[rt] = m_new;
          float psum = 0.f;
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            const float p = ((okbits >> e) & 1u) ? __builtin_amdgcn_exp2f(sv[e] - m_new) : 0.f;
            psum += p;
            pf[rt][e] = (__bf16)p;
          }
          l_run[rt] += psum;
        }
      }
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) {
        union { v4i16 h[2]; bf16x8 v; } vf;
        const char* rowp = vl + 32 * ks * 256 + v_off[dt];
        vf.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4i16*)(rowp));
        vf.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4i16*)(rowp + 16 * 256));
#pragma unroll
        for (int rt = 0; rt < NRT; ++rt)
          o[rt][dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf.v, pf[rt], o[rt][dt], 0, 0, 0);
      }
    }
  };

  int ti = t_begin;
  if (ti < t_end) issue(ti, kA, vA);
  {
    uint64_t my_anc = 0;
    const int tb = dsbd_tree_walk(tr, lane, p_mine, a.max_depth, nullptr, reporter ? a.anc_out : nullptr, &my_anc);
    if (reporter && tb) atomicOr(a.fault, tb);
#pragma unroll
    for (int rt = 0; rt < NRT; ++rt) {
      const int r = row0 + rt * 16 + col;
      const int node = r < R ? r / a.group : 0;
      const unsigned lo = __shfl((unsigned)my_anc, node), hi = __shfl((unsigned)(my_anc >> 32), node);
      anc[rt] = r < R ? ((uint64_t)hi << 32) | lo : 0ull;
    }
  }
  // One barrier per tile: it says that every wave's part of tile ti has landed (each wave waits for its own loads
  // first) and that everybody is done reading the other buffer, into which the next tile is then requested.
  while (ti < t_end) {
    __builtin_amdgcn_s_waitcnt(0x0F70);      // vmcnt(0)
    lds_barrier();
    if (ti + 1 < t_end) issue(ti + 1, kB, vB);
    compute(ti, kA, vA);
    if (++ti >= t_end) break;
    __builtin_amdgcn_s_waitcnt(0x0F70);
    lds_barrier();
    if (ti + 1 < t_end) issue(ti + 1, kA, vA);
    compute(ti, kB, vB);
    ++ti;
  }
  __builtin_amdgcn_s_waitcnt(0x0F70);
  __syncthreads();                           // nobody reads a tile any more: the buffers become the output staging

  // ---- partial results of this split: (m, l) per row, and O^T turned back into rows through the LDS (rows of
  // 512 bytes, 32 rows per array, the 16-byte pieces of a row swizzled by the row number) so that every row leaves
  // as one contiguous write
  constexpr int RPA = SLOTS / 32;            // staged rows per array (512 bytes each): 32 or 16
#pragma unroll
  for (int rt = 0; rt < NRT; ++rt) {
    l_run[rt] += __shfl_xor(l_run[rt], 16);
    l_run[rt] += __shfl_xor(l_run[rt], 32);
    const int rl = wave * ROWS_W + rt * 16 + col;
    const int r = rb * ROWS_B + rl;
    if (r < R && qd == 0) {
      const int node = r / a.group;
      const int head = g * a.group + r % a.group;
      const long long prow = (long long)split * n_rows_total + (long long)(base + node) * a.Hq + head;
      a.part_ml[prow * 2] = m_run[rt];
      a.part_ml[prow * 2 + 1] = l_run[rt];
    }
  }
  // a wave stages its rows in "its" array, RPA rows at a time (all 32 at once with 64-token tiles, else 16 and 16)
  uint4* const st = wave == 0 ? kA : (wave == 1 ? kB : (wave == 2 ? vA : vB));
#pragma unroll
  for (int round = 0; round < ROWS_W / RPA; ++round) {
    if (round > 0) __syncthreads();
#pragma unroll
    for (int rt = 0; rt < NRT; ++rt) {
      if (RPA == 16 && rt != round) continue;
      const int lr = RPA == 16 ? col : rt * 16 + col;        // row within the array
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) {
        union { floatx4 f; uint4 u; } cv;
        cv.f = o[rt][dt];
        st[lr * 32 + ((4 * dt + qd) ^ (col & 7))] = cv.u;
      }
    }
    __syncthreads();
    for (int c = tid; c < 4 * RPA * 32; c += 256) {
      const int w = c / (RPA * 32), lr = (c / 32) % RPA, part = c & 31;
      const int rl = w * ROWS_W + (RPA == 16 ? round * 16 + lr : lr);
      const int r = rb * ROWS_B + rl;
      if (r < R) {
        const int node = r / a.group;
        const int head = g * a.group + r % a.group;
        const long long prow = (long long)split * n_rows_total + (long long)(base + node) * a.Hq + head;
        const uint4* const sr = w == 0 ? kA : (w == 1 ? kB : (w == 2 ? vA : vB));
        const uint4 u = sr[lr * 32 + (part ^ (lr & 7))];
        *reinterpret_cast<uint4*>(&a.part_o[prow * D + 4 * part]) = u;
      }
    }
  }
}

// Merge the KV splits of every (node, head) row: out = sum_s 2^(m_s-M) O_s / sum_s 2^(m_s-M) l_s.
template <int D>
__global__ __launch_bounds__(256) void forest_attention_combine_kernel(int n_rows_total, int nsplit,
                                                                       const float* __restrict__ part_o,
                                                                       const float* __restrict__ part_ml,
                                                                       __bf16* __restrict__ out, float* __restrict__ lse) {
  constexpr int QPR = D / 4;                 // float4 quads per row
  const long long gid = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  const long long row = gid / QPR;
  const int quad = (int)(gid % QPR);
  if (row >= n_rows_total) return;
  // Eight splits at a time with all their loads in flight (a loop of one load and one use per split is bound by
  // memory latency); the running reference M is raised batch by batch.
  float M = NEG_BIG, L = 0.f;
  floatx4 acc = {0.f, 0.f, 0.f, 0.f};
  for (int s0 = 0; s0 < nsplit; s0 += 8) {
    float2 ml[8];
    floatx4 v[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const long long prow = (long long)min(s0 + j, nsplit - 1) * n_rows_total + row;
      ml[j] = *reinterpret_cast<const float2*>(&part_ml[prow * 2]);
      v[j] = *reinterpret_cast<const floatx4*>(&part_o[prow * D + 4 * quad]);
    }
    float Mb = M;
#pragma unroll
    for (int j = 0; j < 8; ++j)
      if (s0 + j < nsplit) Mb = fmaxf(Mb, ml[j].x);
    const float keep = exp2f(M - Mb);                   // 1 when the reference stays
    L *= keep; acc *= keep; M = Mb;
#pragma unroll
    for (int j = 0; j < 8; ++j)
      if (s0 + j < nsplit) {
        const float w = exp2f(ml[j].x - M);
        L += w * ml[j].y;
        acc += w * v[j];
      }
  }
  const float inv = L > 0.f ? 1.f / L : 0.f;
  union { __bf16 h[4]; uint2 u; } pk;
#pragma unroll
  for (int i = 0; i < 4; ++i) pk.h[i] = (__bf16)(acc[i] * inv);
  *reinterpret_cast<uint2*>(&out[row * D + 4 * quad]) = pk.u;
  if (lse && quad == 0) lse[row] = (M + log2f(L)) * 0.6931471805599453f;
}

// ------------------------------------------------------------------------------------------------ host side
namespace {

struct AttnPlan {
  int nrt, rw, tw, rows_block, n_rowblocks, nsplit;
  bool shared;      // LDS-shared K/V tiles (many rows per stream) instead of wave-private streams
  int step;         // tokens per unit of split work
};

AttnPlan make_plan(const dsbd_forest* f, const dsbd_kv* kv, int Hq, int Hkv) {
  AttnPlan p;
  const int group = Hq / Hkv;
  const int rmax = f->max_tree_nodes * group;
  p.shared = false;
  p.step = STEP;
  if (rmax <= 16) { p.nrt = 1; p.rw = 1; p.tw = 4; }
  else if (rmax <= 32) { p.nrt = 2; p.rw = 1; p.tw = 4; }
  else { p.nrt = 2; p.rw = 4; p.tw = 1; p.shared = true; p.step = 64; }   // 128 rows per workgroup
  if (p.shared && dsbd_knobs().attn_waves8) { p.nrt = 1; p.rw = 8; }   // tuning knob: 8 waves x 16 rows
  p.rows_block = 16 * p.nrt * p.rw;
  p.n_rowblocks = (rmax + p.rows_block - 1) / p.rows_block;
  // enough workgroups to fill the chip (two per compute unit are resident; measured on 8 beams x 32 heads with 2048
  // prefix tokens: 2 splits 46.7 us, 4 splits 50.3 us, 1 split 50.5 us), but at least two steps per wave and split
  const long long units = (long long)f->n_trees * Hkv * p.n_rowblocks;
  const int steps = (kv->max_len + p.step - 1) / p.step + 2;
  int by_steps = steps / (2 * p.tw);
  if (by_steps < 1) by_steps = 1;
  int want = (int)((512 + units - 1) / units);
  if (want < 1) want = 1;
  // the split partials (rows x D fp32, written and read once) should stay a small fraction of the K/V bytes
  int by_traffic = kv->max_len / (8 * rmax);
  if (by_traffic < 1) by_traffic = 1;
  p.nsplit = want < by_steps ? want : by_steps;
  if (p.nsplit > by_traffic) p.nsplit = by_traffic;
  if (p.nsplit > 64) p.nsplit = 64;
  {      // tuning knob: KV splits per (tree, KV head, row block)
    const int v = dsbd_knobs().attn_nsplit;
    if (v >= 1 && v <= 64) p.nsplit = v;
  }
  return p;
}

int32_t check_args(const dsbd_forest* f, const dsbd_kv* kv, int Hq, int Hkv, int D) {
  if (!f || !kv) return DSBD_ERR_INVALID;
  if (f->n_trees < 0 || f->n_nodes < 0 || f->n_prompts < 0) return DSBD_ERR_INVALID;
  if (Hq <= 0 || Hkv <= 0 || Hq % Hkv != 0) return DSBD_ERR_INVALID;
  if (D != 128 && D != 64) return DSBD_ERR_UNSUPPORTED;
  if (f->max_tree_nodes < 1 || f->max_tree_nodes > DSBD_MAX_TREE_NODES) return DSBD_ERR_UNSUPPORTED;
  if (kv->max_len < 0) return DSBD_ERR_INVALID;
  if (kv->token_stride % 8 != 0 || kv->head_stride % 8 != 0) return DSBD_ERR_UNSUPPORTED;
  return DSBD_OK;
}

int32_t check_pointers(const dsbd_forest* f, const dsbd_kv* kv) {
  if (f->n_trees > 0 && (!f->tree_off || !f->parent || !kv->k_ptr || !kv->v_ptr || !kv->len)) return DSBD_ERR_INVALID;
  if ((kv->shared_len != nullptr) != (kv->k_shared_ptr != nullptr) ||
      (kv->shared_len != nullptr) != (kv->v_shared_ptr != nullptr)) return DSBD_ERR_INVALID;
  return DSBD_OK;
}

template <int D, int NRT, int RW, int TW>
void launch_attn(const AttnArgs& a, int grid, hipStream_t stream) {
  dsbd_launch(DSBD_KERNEL_ATTENTION, forest_attention_kernel<D, NRT, RW, TW>, dim3(grid), dim3(256), 0, stream, a);
}

template <int D>
void dispatch_attn(const AttnPlan& p, const AttnArgs& a, int grid, hipStream_t stream) {
  if (p.shared) {
    if constexpr (D == 128) {
      if (p.nrt == 1) {
        dsbd_launch(DSBD_KERNEL_ATTENTION, forest_attention_shared_kernel<D, 8, 1>, dim3(grid), dim3(512), 0, stream, a);
        return;
      }
    }
    if constexpr (D == 128) {
      if (!dsbd_knobs().attn_staged) {     // (knob: the kernel that stages the tiles through registers, for comparison)
        dsbd_launch(DSBD_KERNEL_ATTENTION, forest_attention_dma_kernel<64, 2>, dim3(grid), dim3(256), 0, stream, a);
        return;
      }
    }
    dsbd_launch(DSBD_KERNEL_ATTENTION, forest_attention_shared_kernel<D, 4, 2>, dim3(grid), dim3(256), 0, stream, a);
  } else if (p.nrt == 1) {
    launch_attn<D, 1, 1, 4>(a, grid, stream);
  } else {
    launch_attn<D, 2, 1, 4>(a, grid, stream);
  }
}

}  // namespace

extern "C" size_t dsbd_forest_attention_workspace_bytes(const dsbd_forest* f, const dsbd_kv* kv, int32_t Hq,
                                                        int32_t Hkv, int32_t D) {
  if (check_args(f, kv, Hq, Hkv, D) != DSBD_OK) return 0;
  const AttnPlan p = make_plan(f, kv, Hq, Hkv);
  WorkspaceCarver ws(nullptr);
  ws.take<long long>(4096);
  ws.take<float>((size_t)p.nsplit * f->n_nodes * Hq * D);
  ws.take<float>((size_t)p.nsplit * f->n_nodes * Hq * 2);
  return ws.total() + 256;
}

extern "C" int32_t dsbd_forest_attention(const dsbd_forest* f, const dsbd_kv* kv, const void* q, const void* k_tree,
                                         const void* v_tree, int32_t Hq, int32_t Hkv, int32_t D, float scale,
                                         void* out, float* lse, uint64_t* anc_mask_out, void* workspace,
                                         size_t workspace_bytes, int32_t* fault, void* stream_) {
  int32_t rc = check_args(f, kv, Hq, Hkv, D);
  if (rc != DSBD_OK) return rc;
  if (!fault) return DSBD_ERR_INVALID;
  if (f->n_nodes == 0 || f->n_trees == 0) return DSBD_OK;
  rc = check_pointers(f, kv);
  if (rc != DSBD_OK) return rc;
  if (!q || !k_tree || !v_tree || !out || !workspace) return DSBD_ERR_INVALID;
  if ((reinterpret_cast<uintptr_t>(q) | reinterpret_cast<uintptr_t>(k_tree) | reinterpret_cast<uintptr_t>(v_tree) |
       reinterpret_cast<uintptr_t>(out)) & 15)
    return DSBD_ERR_INVALID;
  if (workspace_bytes < dsbd_forest_attention_workspace_bytes(f, kv, Hq, Hkv, D)) return DSBD_ERR_WORKSPACE;
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  const AttnPlan p = make_plan(f, kv, Hq, Hkv);

  char* wbase = reinterpret_cast<char*>(dsbd_align_up(reinterpret_cast<uintptr_t>(workspace), 256));
  WorkspaceCarver ws(wbase);
  long long* trace = ws.take<long long>(4096);
  float* part_o = ws.take<float>((size_t)p.nsplit * f->n_nodes * Hq * D);
  float* part_ml = ws.take<float>((size_t)p.nsplit * f->n_nodes * Hq * 2);
  AttnArgs a;
  a.tree_off = f->tree_off; a.parent = f->parent;
  a.max_tree_nodes = f->max_tree_nodes; a.max_depth = f->max_depth; a.anc_out = anc_mask_out;
  a.k_ptr = kv->k_ptr; a.v_ptr = kv->v_ptr; a.len = kv->len;
  a.k_shared_ptr = kv->k_shared_ptr; a.v_shared_ptr = kv->v_shared_ptr; a.shared_len = kv->shared_len;
  a.token_stride = kv->token_stride; a.head_stride = kv->head_stride;
  a.q = static_cast<const __bf16*>(q); a.k_tree = static_cast<const __bf16*>(k_tree);
  a.v_tree = static_cast<const __bf16*>(v_tree);
  a.n_nodes = f->n_nodes; a.Hq = Hq; a.Hkv = Hkv; a.group = Hq / Hkv;
  const float sc = scale > 0.f ? scale : 1.0f / sqrtf((float)D);
  a.scale_log2 = sc * 1.4426950408889634f;
  a.nsplit = p.nsplit; a.n_rowblocks = p.n_rowblocks; a.max_len = kv->max_len;
  a.part_o = part_o; a.part_ml = part_ml; a.fault = fault;
  a.trace = dsbd_knobs().attn_trace ? trace : nullptr;

  const long long grid = (long long)f->n_trees * Hkv * p.n_rowblocks * p.nsplit;
  if (grid > 0x7fffffffLL) return DSBD_ERR_UNSUPPORTED;
  if (D == 128) dispatch_attn<128>(p, a, (int)grid, stream);
  else dispatch_attn<64>(p, a, (int)grid, stream);
  DSBD_HIP_LAUNCH_CHECK();

  const long long n_rows_total = (long long)f->n_nodes * Hq;
  const long long threads = n_rows_total * (D / 4);
  const int cgrid = (int)((threads + 255) / 256);
  if (D == 128)
    hipLaunchKernelGGL(forest_attention_combine_kernel<128>, dim3(cgrid), dim3(256), 0, stream, (int)n_rows_total,
                       p.nsplit, part_o, part_ml, static_cast<__bf16*>(out), lse);
  else
    hipLaunchKernelGGL(forest_attention_combine_kernel<64>, dim3(cgrid), dim3(256), 0, stream, (int)n_rows_total,
                       p.nsplit, part_o, part_ml, static_cast<__bf16*>(out), lse);
  DSBD_HIP_LAUNCH_CHECK();
  return DSBD_OK;
}
