/*
 * dsbd.h - C ABI of the multi-tree (forest) parallel verification step of dynamic-width
 * speculative beam decoding, for AMD MI355X (gfx950).
 *
 * One decoding iteration hands this library a draft forest (one token tree per input beam),
 * the large model's per-beam key/value caches, and the large/small models' logits at every
 * forest node.  The library
 *   1. runs forest attention: every node attends to its own beam's cache plus its tree
 *      ancestors (paper Section 3.3, "Forest-based Parallel Decoding");
 *   2. verifies the forest layer by layer (paper Section 3.1 "Details", Algorithm 1) with the
 *      fixed or the dynamic layer width (Section 3.2, Eq. 1-6);
 *   3. turns the verification result into the next iteration's beam set (Algorithm 1's return
 *      value; Section 3.3 last paragraph; Section 3.4 for the one-beam variant);
 *   4. updates the key/value caches to follow that beam set (Section 3.3 last paragraph).
 *
 * Conventions
 *   - Every array argument is a DEVICE pointer owned by the caller unless marked "host".
 *     The structs themselves are host memory, read during the call only.
 *   - The library allocates no device memory and keeps no state between calls (apart from the measurement
 *     hook at the end of this header, the tuning knobs it reads once, and one extra stream with two events per
 *     device that dsbd_verify_forest creates at its first call or dsbd_init() creates).  Scratch memory comes
 *     from the caller's `workspace` (device, 256-byte aligned), at least as large as the
 *     matching dsbd_*_workspace_bytes() says.  Its contents need not be initialised.
 *   - `stream` is a hipStream_t passed as void*.  Calls only enqueue work; outputs are valid
 *     once the stream has been synchronised.  No call synchronises the device.
 *   - Return value: DSBD_OK or a negative DSBD_ERR_* for problems visible on the host
 *     (null pointers, sizes, unsupported shapes, workspace too small, HIP launch errors).
 *     Nothing is enqueued when an error is returned (one exception: see dsbd_verify_forest).
 *   - Problems only visible in device data are OR-ed into the device word `*fault`
 *     (DSBD_FAULT_* bits) and never cause out-of-bounds accesses; the caller clears the word.
 */
#ifndef DSBD_H
#define DSBD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define DSBD_OK               0
#define DSBD_ERR_INVALID     (-1)   /* null pointer, negative size, Hq % Hkv != 0, ...              */
#define DSBD_ERR_UNSUPPORTED (-2)   /* D not 128 or 64, tree bound above 64 nodes, V < 1 or > 2^30, ... */
#define DSBD_ERR_WORKSPACE   (-3)   /* workspace smaller than dsbd_*_workspace_bytes()              */
#define DSBD_ERR_HIP         (-4)   /* HIP runtime reported an error at launch                      */

#define DSBD_FAULT_TOPOLOGY       1 /* parent outside its tree / not before the child / bad root    */
#define DSBD_FAULT_TOKEN          2 /* token id outside [0, V)                                      */
#define DSBD_FAULT_NONFINITE      4 /* NaN or +Inf logit; -Inf (a masked token) in a whole row or at */
                                    /* a drafted token; a layer without an input beam of finite     */
                                    /* likelihood under one of the models                           */
#define DSBD_FAULT_ZERO_RESIDUAL  8 /* a residual distribution had no mass                          */
#define DSBD_FAULT_BOUNDS        16 /* a host-declared bound (max_*) is exceeded by the device data */
#define DSBD_FAULT_SYNC_TIMEOUT  32 /* internal grid synchronisation gave up                        */

/* node_status codes written by dsbd_verify_forest */
#define DSBD_NOT_REACHED 0          /* deeper than the last verified layer                          */
#define DSBD_ACCEPTED    1
#define DSBD_REJECTED    2          /* failed its test, or left over once the layer was full         */
#define DSBD_PRUNED      3          /* its parent was not accepted (Algorithm 1, pruning step)       */
#define DSBD_ROOT        4          /* an input beam                                                */

/*
 * Draft forest (Section 3.1 "Overview"): n_trees token trees, one per input beam, the trees of a
 * prompt adjacent.  Nodes of a tree are contiguous, the first node of a tree is its root (the
 * input beam's last token) and parent[i] < i (depth-first order as in the forest-attention
 * figure satisfies this, so does breadth-first order).
 */
typedef struct dsbd_forest {
  int32_t n_prompts, n_trees, n_nodes;
  const int32_t* tree_prompt;   /* [n_trees]   prompt of each tree, non-decreasing, 0..n_prompts-1    */
  const int32_t* tree_off;      /* [n_trees+1] first node of each tree; tree_off[n_trees] = n_nodes   */
  const int32_t* parent;        /* [n_nodes]   global index of the parent, -1 at a root               */
  const int32_t* token;         /* [n_nodes]   token id at the node (verify only; may be NULL for attention) */
  const int32_t* draft_rank;    /* [n_nodes] or NULL: order in which the draft stage drew the nodes   */
                                /*   of a layer; a layer is verified in ascending (rank, node index). */
                                /*   The correctness theorem needs the draw order (iid drafts).      */
  /* host-side bounds on the device data, checked on the device (DSBD_FAULT_BOUNDS): */
  int32_t max_tree_nodes;       /* >= nodes of the largest tree; at most 64                           */
  int32_t max_depth;            /* >= depth of the deepest node (roots have depth 0)                  */
  int32_t max_prompt_trees;     /* >= trees of the widest prompt                                      */
} dsbd_forest;

/*
 * Per-beam prefix key/value caches (Section 3.3: one cache per input beam), bf16.
 * The prefix of tree b is an optional segment shared with other beams (k_shared_ptr[b], first
 * shared_len[b] tokens) followed by the beam's own segment (k_ptr[b], len[b] tokens).
 * Element (token t, kv-head g, channel d) of a segment lives at ptr[t*token_stride + g*head_stride + d]
 * (strides in elements; covers [L,Hkv,D] and [Hkv,L,D]).  The two strides are common to ALL segments of all
 * trees (head-major caches therefore share one capacity: head_stride = capacity * D), and the library cannot
 * check them against the allocations: the caller guarantees that t*token_stride + g*head_stride + d stays inside
 * every segment for t < its length and g < Hkv.  The root token's K/V is NOT part of
 * the prefix: it is row tree_off[b] of k_tree / v_tree.
 */
typedef struct dsbd_kv {
  const void* const* k_ptr;         /* [n_trees] device array of device pointers                      */
  const void* const* v_ptr;         /* [n_trees]                                                      */
  const int32_t*     len;           /* [n_trees] tokens in the own segment (>= 0)                     */
  const void* const* k_shared_ptr;  /* [n_trees] or NULL                                              */
  const void* const* v_shared_ptr;  /* [n_trees] or NULL                                              */
  const int32_t*     shared_len;    /* [n_trees] or NULL                                              */
  int64_t token_stride, head_stride;
  int32_t max_len;                  /* host bound: >= shared_len[b] + len[b] for every tree           */
} dsbd_kv;

size_t dsbd_forest_attention_workspace_bytes(const dsbd_forest* forest, const dsbd_kv* prefix,
                                             int32_t Hq, int32_t Hkv, int32_t D);

/*
 * Forest attention (Section 3.3 and the forest-attention figure): for node n of tree b and query
 * head h, softmax over {all prefix positions of beam b} U {tree rows of n's ancestors and n itself}
 * of scale * q.k, applied to V.  Query head h reads KV head h / (Hq/Hkv).
 *   q               [n_nodes,Hq,D]  bf16
 *   k_tree, v_tree  [n_nodes,Hkv,D] bf16, row n = key/value of forest node n
 *   scale           <= 0 selects 1/sqrt(D)
 *   out             [n_nodes,Hq,D]  bf16
 *   lse             [n_nodes,Hq]    f32 natural-log sum of exp of the scaled scores, or NULL
 *   anc_mask_out    [n_nodes]       u64 or NULL; bit j = j-th node of the same tree is an ancestor or the node itself
 * Supported: D = 128 or 64, Hq % Hkv == 0, trees of at most 64 nodes.
 */
int32_t dsbd_forest_attention(const dsbd_forest* forest, const dsbd_kv* prefix,
                              const void* q, const void* k_tree, const void* v_tree,
                              int32_t Hq, int32_t Hkv, int32_t D, float scale,
                              void* out, float* lse, uint64_t* anc_mask_out,
                              void* workspace, size_t workspace_bytes, int32_t* fault, void* stream);

/* Verification parameters (Algorithm 1 inputs; Eq. 5-6). */
typedef struct dsbd_params {
  int32_t W_L;     /* beam width; <= 0: every prompt uses its own number of input beams             */
  int32_t W_min;   /* floor of the dynamic width (Eq. 5), >= 1                                      */
  int32_t W_cap;   /* capacity of the per-prompt output arrays; also caps every layer's width       */
  float   t;       /* threshold of Eq. 6 in [0,1]; t < 0 selects the fixed width W_L for all layers */
  /* Warping operation T of beam sampling (Section 2.1; Section 3.1 "Details": p_beam = T o p/P), applied to   */
  /* both joints over I x V in every layer and to p_beam of the bonus layer.  Entries are ranked by value,     */
  /* equal values by lower flat index (beam-major, token-minor).                                               */
  int32_t top_k;   /* keep the top_k largest entries; 0: keep all.  1..32 supported; > 32: UNSUPPORTED         */
  float   top_p;   /* of those kept, the shortest leading part whose share of their mass exceeds top_p, then   */
                   /* renormalise; 0 or >= 1: no cut (a zeroed struct means no warping).  A value in (0,1)     */
                   /* needs top_k >= 1 (else UNSUPPORTED); < 0: INVALID                                        */
} dsbd_params;

/* Inputs of the verification that are not part of the forest. Lmax = forest->max_depth. */
typedef struct dsbd_verify_in {
  int32_t V;                       /* vocabulary size                                                */
  const float*  logits_target;     /* [n_nodes,V] large model's logits at every node (row-major);    */
                                   /*   -Inf = a masked token (probability 0); a row needs one finite */
                                   /*   logit and a drafted token a finite logit in its parent's row  */
                                   /*   (both models); NaN, +Inf, a row of -Inf only and a masked     */
                                   /*   drafted token raise DSBD_FAULT_NONFINITE                      */
  const float*  logits_draft;      /* [n_nodes,V] small model's logits                               */
  const double* beam_logp_target;  /* [n_trees] stored log-likelihood of each input beam under p      */
  const double* beam_logp_draft;   /* [n_trees] ... under q (Section 2.1: beam sampling stores them). */
                                   /*   -Inf: a beam of probability 0 under that model (with DIFFERENT */
                                   /*   masks in the two models an output beam can come back with     */
                                   /*   out_logp_draft = -Inf: a token drawn from the residual that   */
                                   /*   the small model masks).  A layer whose input beams ALL have   */
                                   /*   -Inf under one model has no joint: DSBD_FAULT_NONFINITE, as   */
                                   /*   for NaN and +Inf                                              */
  const float*  u_accept;          /* [n_nodes]            uniform in [0,1) for the node's accept test */
  const float*  u_resid;           /* [n_prompts,Lmax+2]   uniform for the residual sample of layer l  */
  const float*  u_fill;            /* [n_prompts,Lmax+2,W_cap] uniforms for the p_beam samples of layer l */
} dsbd_verify_in;

/* Outputs of the verification. */
typedef struct dsbd_verify_out {
  uint8_t* node_status;        /* [n_nodes] DSBD_* status codes                                      */
  float*   lse_target;         /* [n_nodes] log-sum-exp of the node's target logits                  */
  float*   lse_draft;          /* [n_nodes]                                                          */
  float*   node_logp_target;   /* [n_nodes] log p(token[n] | parent[n]); 0 at roots                  */
  float*   node_logp_draft;    /* [n_nodes]                                                          */
  int32_t* l_last;             /* [n_prompts] layer that produced the output beams (1..gamma+1)      */
  int32_t* layer_width;        /* [n_prompts,Lmax+2] W_L^(l) used at layer l (index 0: input beams)  */
  int32_t* n_out;              /* [n_prompts] number of output beams                                 */
  int32_t* out_parent;         /* [n_prompts,W_cap] forest node the output beam extends              */
  int32_t* out_token;          /* [n_prompts,W_cap] its new token                                    */
  int32_t* out_node;           /* [n_prompts,W_cap] the accepted draft node, or -1 if sampled        */
  double*  out_logp_target;    /* [n_prompts,W_cap] cumulative log-likelihood of the output beam (p) */
  double*  out_logp_draft;     /* [n_prompts,W_cap] ... under q                                      */
  int32_t* near_tie_count;     /* [n_prompts] accept tests with |ratio - u| <= 1e-6                  */
} dsbd_verify_out;

size_t dsbd_verify_forest_workspace_bytes(const dsbd_forest* forest, int32_t V, const dsbd_params* params);

/*
 * Layer-wise verification of the draft forest (Algorithm 1; Section 3.1 "Details"; Section 3.2):
 * per-node vocabulary softmax of both models, beam-sampling joints p_beam / q_beam over the
 * layer's input beams, sequential accept test r <= p'/q_beam with the residual update
 * p' <- norm(max(0, p' - q_beam)) on rejection and p' <- p_beam on acceptance, early stop at
 * W_L^(l) accepted beams, residual + p_beam sampling when a layer falls short, and the bonus
 * layer when every layer passes.  Decisions are taken in fp64.
 *   - Limits: at most 64 input beams, 512 forest nodes and W_cap <= 64 per prompt.  Any number of prompts: when
 *     they need more workgroups than the device holds at once, the layer kernel is launched for one group of
 *     prompts after the other (Algorithm 1 runs per prompt).
 *   - Two kernels run side by side: the layer kernel on `stream`, and the pass over all logits that produces the
 *     per-node outputs (lse_*, node_logp_*) on a second stream that the library creates once per device; the second
 *     stream starts after everything `stream` holds at the time of the call and `stream` continues only when both
 *     kernels are done, so the caller sees ordinary stream semantics.  If all four per-node outputs are NULL the
 *     pass is left out; NaN and +Inf logits are then reported only for the rows of beams that enter a layer, and
 *     the two misuses of -Inf (a row of nothing else, a masked drafted token) not at all.
 *   - The layer kernel's workgroups wait for each other, so it needs its share of the device while it runs.
 *     Verifications on DIFFERENT streams are kept apart by the library: the first call that arrives on another
 *     stream than the one before waits for the device to drain (once per device and process), and from then on
 *     every layer kernel is ordered behind the previous one by an event (6 us per call, which callers that stay on
 *     one stream never pay).  A stream under graph capture: the call can be recorded (its second stream joins the
 *     capture through the fork and join events; a one-thread kernel in front of the layer kernel counts the replays in
 *     the workspace, so that every replay's exchange slots are told apart from the previous one's, which is why the
 *     workspace must be the same memory at every replay), but it records nothing outside the capture: keep replays
 *     apart from other verifications yourself.  Also not covered: dsbd_verify_forest_static() before the
 *     library's second stream exists, and other processes on the device.  Foreign kernels that occupy compute
 *     units only delay the layer kernel; every wait in it is bounded (3 s by default) and ends in
 *     DSBD_FAULT_SYNC_TIMEOUT with unusable outputs, never in a hang.
 *   - If a launch fails after the first kernel has been enqueued the call returns DSBD_ERR_HIP with that kernel
 *     already on the stream (every other error is reported before anything is enqueued).
 *   - The workspace must not be shared by calls that may overlap.
 *   - logits_target == logits_draft together with beam_logp_target == beam_logp_draft (one model in both roles,
 *     as dsbd_draft_layer passes them) is recognised: the joint is then formed once; the results are those of two
 *     equal models.
 */
int32_t dsbd_verify_forest(const dsbd_forest* forest, const dsbd_verify_in* in, const dsbd_params* params,
                           const dsbd_verify_out* out,
                           void* workspace, size_t workspace_bytes, int32_t* fault, void* stream);

/*
 * dsbd_verify_forest for callers that cannot allocate device memory: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Same arguments, results and error behaviour as dsbd_verify_forest, minus
 * the workspace: it lives in a device array of dsbd_verify_forest_static_capacity() bytes (32 MiB) that is part of
 * the library's image (every GPU the library runs on holds its own copy until the process ends).  A problem whose
 * dsbd_verify_forest_workspace_bytes() exceeds the capacity is refused with DSBD_ERR_WORKSPACE and nothing is
 * enqueued.  The call allocates nothing: no device memory, no stream, no event; the statistics pass runs beside the
 * layer kernel only if an earlier ordinary call or dsbd_init() has already created the library's second stream on
 * this device, otherwise in front of it on the caller's stream.  Nothing in the array has to be cleared between
 * calls (exchange slots are told apart by a per-launch tag).  All calls on one GPU share that GPU's array: calls
 * that overlap in time on one GPU (different streams, or host threads) race and give undefined results.
 *
 * dsbd_init() (optional): resolves the array's address and creates the second stream for the CURRENT device, so
 * that the first call after it allocates nothing either.  Returns DSBD_OK or DSBD_ERR_HIP.
 */
int32_t dsbd_init(void);
size_t dsbd_verify_forest_static_capacity(void);
int32_t dsbd_verify_forest_static(const dsbd_forest* forest, const dsbd_verify_in* in, const dsbd_params* params,
                                  const dsbd_verify_out* out, int32_t* fault, void* stream);

/* Next beam set. */
typedef struct dsbd_next_beams {
  int32_t* n_next;      /* [n_prompts]                                                               */
  int32_t* src_tree;    /* [n_prompts,W_cap] tree (input beam) whose cache the new beam continues     */
  int32_t* src_out;     /* [n_prompts,W_cap] index of the verification output beam it came from       */
  int32_t* path_len;    /* [n_prompts,W_cap] number of forest nodes on the path root..out_parent      */
  int32_t* path;        /* [n_prompts,W_cap,Lmax+1] those nodes, root first (tree rows to append to   */
                        /*   the cache); unused entries -1                                            */
  int32_t* token;       /* [n_prompts,W_cap] last token of the new beam                               */
  double*  logp_target; /* [n_prompts,W_cap]                                                          */
  double*  logp_draft;  /* [n_prompts,W_cap]                                                          */
} dsbd_next_beams;

/*
 * Select the beams of the next iteration from the verification outputs (Algorithm 1 returns the
 * beams of layer l_last; Section 3.3: the caches kept are those the output beams descend from).
 * keep_one != 0: keep only the output beam with the highest cumulative target log-likelihood
 * (lowest perplexity; ties to the lowest index), so a single cache survives (Section 3.4).  The comparison is that
 * of the fp64 values in out_logp_target: likelihoods of different beams that are equal in exact arithmetic may differ
 * there in the last bit.
 * W_cap and Lmax must be the values used for dsbd_verify_forest.
 */
int32_t dsbd_select_beams(const dsbd_forest* forest, const dsbd_verify_out* verified, int32_t W_cap,
                          int32_t keep_one, const dsbd_next_beams* next, int32_t* fault, void* stream);

/*
 * Verification and selection in one call (Algorithm 1 with its return statement; Section 3.3, last paragraph;
 * Section 3.4 for keep_one): dsbd_verify_forest followed by dsbd_select_beams with W_cap = params->W_cap, same
 * arguments, same results in `out` and `next`, same error behaviour, one `fault` word for both.  With keep_one == 0
 * no selection kernel is launched: the workgroup of the layer kernel that writes an output beam also writes the
 * beam's entry of the plan (the tree whose cache it continues, the path of forest nodes from the root).  With
 * keep_one != 0 the single surviving beam is chosen among all output beams of a prompt, so the selection kernel
 * runs behind the verification on `stream`.  An empty forest writes nothing, as in dsbd_verify_forest.
 */
int32_t dsbd_verify_forest_select(const dsbd_forest* forest, const dsbd_verify_in* in, const dsbd_params* params,
                                  const dsbd_verify_out* out, int32_t keep_one, const dsbd_next_beams* next,
                                  void* workspace, size_t workspace_bytes, int32_t* fault, void* stream);

/*
 * Destination caches of the next iteration's beams, one per slot (p, j) of the next-beam plan, in the layout
 * (strides) of the source caches.  Only the own segment is written; a segment shared by the beams of a prompt
 * stays where it is.
 */
typedef struct dsbd_kv_dst {
  void* const* k_ptr;   /* [n_prompts*W_cap] device array of device pointers (entries of unused slots are ignored) */
  void* const* v_ptr;   /* [n_prompts*W_cap]                                                           */
  int32_t*     len;     /* [n_prompts*W_cap] out: tokens of the new own segment, 0 in unused slots     */
  int32_t      capacity;/* tokens every destination buffer can hold                                    */
} dsbd_kv_dst;

/*
 * Physical cache update (Section 3.3, last paragraph: the caches follow the output beams; Section 3.4: one
 * cache in the memory-reduced variant).  For every next beam (p, j), j < next->n_next[p]: destination (p, j) :=
 * own segment of tree next->src_tree[p,j] (src->len tokens), followed by the rows k_tree / v_tree [n_nodes,Hkv,D]
 * of the nodes next->path[p,j,0 .. path_len) (root first).  The output beam's own last token is the root of the
 * next iteration's tree and gets its row in the next forward pass.  Bit-exact copies of bf16 data.
 *   - A destination pointer equal to its source pointer means "continue in place": only the tree rows are appended
 *     (at most one next beam per source tree can do that).  Apart from this, destination buffers must not overlap
 *     any source segment or each other: the copies run concurrently.
 *   - Device-side problems: a plan entry outside the forest (DSBD_FAULT_TOPOLOGY), a new length above
 *     dst->capacity, a null or misaligned (16 bytes) pointer (DSBD_FAULT_BOUNDS); the affected destination gets
 *     length 0 (or, for a bad path node, that row is skipped) and nothing is written out of bounds.
 * W_cap and forest->max_depth must be the values used for dsbd_select_beams.
 */
int32_t dsbd_commit_kv(const dsbd_forest* forest, const dsbd_kv* src, const void* k_tree, const void* v_tree,
                       int32_t Hkv, int32_t D, const dsbd_next_beams* next, int32_t W_cap,
                       const dsbd_kv_dst* dst, int32_t* fault, void* stream);

/*
 * Draft stage, one step (Section 3.1 "Overview": the small model performs beam sampling of width W_S for gamma
 * steps; "Details": a draft beam of the next layer is a sample of q_beam = T o q/Q over (beams of the current
 * layer) x V, the W_S draft beams of a layer drawn independently).  The beams of the current layer are rows:
 * the input beams for the first step, the W_S draws of the step before afterwards.
 */
typedef struct dsbd_draft_in {
  int32_t n_prompts;
  int32_t n_beams;                 /* rows of the current layer, all prompts                                 */
  int32_t max_prompt_beams;        /* host-side bound: most beams of one prompt (<= 64)                      */
  int32_t V;
  const int32_t* beam_off;         /* [n_prompts+1] device: beams of prompt p are rows beam_off[p] .. beam_off[p+1]-1 */
  const float*   logits_draft;     /* [n_beams,V] small model's logits at those beams (-Inf = a masked token, */
                                   /*   never drawn; a row needs one finite logit)                            */
  const double*  beam_logp_draft;  /* [n_beams] their stored log-likelihoods under the small model (-Inf: a   */
                                   /*   beam that is never continued; finite for one beam of every prompt)    */
  const float*   u;                /* [n_prompts,W_S] uniforms in [0,1), one per draw                        */
} dsbd_draft_in;

typedef struct dsbd_draft_out {    /* device arrays [n_prompts,W_S]; draw j of prompt p at p*W_S + j          */
  int32_t* parent;                 /* row (0 .. n_beams-1) of the beam the draw continues                    */
  int32_t* token;
  double*  logp_draft;             /* log-likelihood of the new beam under the (unwarped) small model        */
} dsbd_draft_out;

size_t dsbd_draft_layer_workspace_bytes(const dsbd_draft_in* in, int32_t W_S, int32_t top_k, float top_p);

/*
 * W_S independent inverse-CDF draws per prompt from q_beam over (the prompt's beams) x V, flat order beam-major /
 * token-minor, warped by top_k / top_p as in dsbd_params (0 / 1: no warping).  Decisions in fp64; the same
 * kernels as the verification's sampling of its additional layer.  W_S in 1..64.  A prompt without beams gets
 * parent = token = -1.  Faults as for dsbd_verify_forest (non-finite logits, inconsistent beam_off).
 */
int32_t dsbd_draft_layer(const dsbd_draft_in* in, int32_t W_S, int32_t top_k, float top_p,
                         const dsbd_draft_out* out, void* workspace, size_t workspace_bytes,
                         int32_t* fault, void* stream);

/*
 * Lays the sampled layers out as the draft forest (Section 3.1 "Overview": one tree per input beam, every layer
 * from the second on holds the W_S intermediate beams of a step).  Layer l = 1..gamma: draw j of prompt p is row
 * p*W_S + j with parent row layer_parent[(l-1)*n_prompts*W_S + p*W_S + j] in layer l-1 (a row of
 * dsbd_draft_layer's input at that step) and token layer_token[...].
 * Layout written: trees contiguous in input-beam order; inside a tree the root, then its nodes by (layer, draw
 * index), so parent < child; draft_rank = draw index within the layer (the order dsbd_verify_forest must test a
 * layer's candidates in); n_nodes = n_roots + gamma*n_prompts*W_S.
 * Device-side problems (fault bits): a parent row outside its prompt's rows of the layer before
 * (DSBD_FAULT_TOPOLOGY; the node is hung under the first valid row), a tree of more than 64 nodes or a prompt of
 * more than 512 (DSBD_FAULT_BOUNDS; the arrays are still consistent, but the forest is not usable by the other
 * calls).
 */
typedef struct dsbd_forest_out {   /* device arrays, caller-allocated */
  int32_t* tree_prompt;            /* [n_roots]                                                              */
  int32_t* tree_off;               /* [n_roots+1]                                                            */
  int32_t* parent;                 /* [n_nodes]                                                              */
  int32_t* token;                  /* [n_nodes]                                                              */
  int32_t* draft_rank;             /* [n_nodes]                                                              */
  int32_t* node_of_root;           /* [n_roots] forest node of every input beam (= tree_off[b])              */
  int32_t* node_of;                /* [gamma*n_prompts*W_S] forest node of every draw, layer-major           */
  int32_t* max_tree_nodes;         /* [1] nodes of the largest tree                                          */
} dsbd_forest_out;

int32_t dsbd_build_forest(int32_t n_prompts, int32_t n_roots, int32_t gamma, int32_t W_S,
                          const int32_t* root_off,      /* [n_prompts+1] device: input beams of prompt p    */
                          const int32_t* root_token,    /* [n_roots] device or NULL (roots then get token 0) */
                          const int32_t* layer_parent,  /* [gamma,n_prompts*W_S] device                      */
                          const int32_t* layer_token,   /* [gamma,n_prompts*W_S] device                      */
                          const dsbd_forest_out* out, int32_t* fault, void* stream);

/*
 * Tuning overrides (no counterpart in the paper).  The library reads its DSBD_* environment variables (numbers of
 * KV splits and of workgroups per prompt, chunk sizes, the bound of the layer kernel's waits, test hooks) ONCE per
 * process, at the first call that needs them; dsbd_reload_knobs() reads them again.  Host call, no GPU work.
 */
void dsbd_reload_knobs(void);

/*
 * Measurement hook (no counterpart in the paper).  dsbd_timing_enable(kernel, capacity) makes the
 * library record a pair of HIP events around every launch of ONE of its kernels, on the stream the
 * kernel is launched on, for up to `capacity` launches; dsbd_timing_collect() waits for the recorded
 * events, writes the elapsed milliseconds of each launch to the HOST array `ms` (at most max_n) and
 * returns how many it wrote (negative: DSBD_ERR_*), then starts over.  kernel = 0 switches it off and
 * frees the events.  Not thread-safe; meant for benchmarks.
 */
#define DSBD_KERNEL_ATTENTION     1   /* forest attention main kernel (streams K/V)            */
#define DSBD_KERNEL_VOCAB_STATS   2   /* per-node vocabulary softmax statistics (streams logits) */
#define DSBD_KERNEL_VERIFY_LAYERS 3   /* persistent layer-by-layer verification                */
#define DSBD_KERNEL_KV_COMMIT     4   /* cache update (copies the surviving caches)             */
int32_t dsbd_timing_enable(int32_t kernel, int32_t capacity);
int32_t dsbd_timing_collect(float* ms, int32_t max_n);

/*
 * Measurement aid (no counterpart in the paper): a plain streaming read of `bytes` (>= 1 MiB, 16-byte aligned DEVICE
 * buffer, left unchanged) with the access pattern of the library's bandwidth-bound kernels, `reps` times between HIP
 * events on `stream`; the shortest time in milliseconds goes to the HOST word best_ms.  It says what fraction of the
 * datasheet bandwidth a pure read reaches on the box at hand.  Blocks until the runs are done.
 */
int32_t dsbd_stream_read_probe(const void* buf, size_t bytes, int32_t reps, float* best_ms, void* stream);

/* Library version and the offload architecture it was built for. */
const char* dsbd_version(void);

#ifdef __cplusplus
}
#endif
#endif /* DSBD_H */
