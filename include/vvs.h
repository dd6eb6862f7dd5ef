/*
 * vvs.h - C ABI of the MI355X (gfx950) target-model verification pass for speculative decoding of
 * visual autoregressive models.
 *
 * One call of vvs_verify is one "target forward pass" in the sense of the paper's tokens-per-forward
 * metric (Section 5, "Metrics"): a KV-cached decoder-only transformer scores the pending token and N
 * drafted VQ tokens (a chain, or a tree under an ancestor mask: Section 3, "Verification
 * Redundancy") for B prompts, each as a conditional / unconditional row pair, mixes the two logit
 * rows, applies softmax, and runs the accept / resample rule of Section 2 ("Speculative Decoding").
 * vvs_kv_commit then keeps the K/V of the accepted path (Section 4.1: restoring the KV entries
 * re-establishes exact AR conditioning).
 *
 * Notation: p = target distribution, q = draft distribution (the paper prints the two letters the
 * other way round; the rule is the same: accept with probability min(1, target/draft)).
 * B prompts; R = 2B rows, row 2b conditional, row 2b+1 unconditional; N draft nodes numbered 1..N,
 * node 0 = root = the pending token (emitted, K/V not cached yet); T = N + 1; V_eff = logit_hi -
 * logit_lo; S_b = cached length of prompt b.
 *
 * Ownership: the caller allocates every device buffer (KV cache, workspace, packed weights, inputs,
 * outputs), sized by vvs_query_sizes; the library never allocates or frees device memory and never
 * synchronises the stream, except vvs_create (synchronous: it zero-fills the KV cache and uploads
 * small tables).  Pointers named d_* are DEVICE pointers, h_* are HOST pointers.  Device buffers
 * must stay valid until the work queued on the stream has finished.  Calls on one context must be
 * issued on one stream (or be ordered by the caller).
 *
 * Errors: every function returns a vvs_status; nothing is launched when the status is not VVS_OK
 * (arguments and call order are checked on the host first).  vvs_last_error gives the message.
 */
#ifndef VVS_H
#define VVS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct vvs_ctx vvs_ctx;        /* opaque host object; owns no device memory */
typedef void* vvs_stream;              /* a hipStream_t (NULL = the default stream) */

typedef enum {
  VVS_OK = 0,
  VVS_EINVAL = -1,   /* bad argument (NULL pointer, malformed tree, value out of range) */
  VVS_ESTATE = -2,   /* call order: verify before prefill, commit without verify, ... */
  VVS_ESIZE = -3,    /* shape not supported / exceeds the sizes the context was created for */
  VVS_EHIP = -4      /* a HIP call failed */
} vvs_status;

enum { VVS_FP32 = 0, VVS_BF16 = 1 };               /* vvs_config.dtype */
enum { VVS_PREFIX_CLASS = 0, VVS_PREFIX_DENSE = 1 }; /* vvs_config.prefix_kind */
enum { VVS_STRICT = 0, VVS_RELAXED = 1 };           /* acceptance mode */
#define VVS_MAX_T 64                                 /* max query tokens per row in one verify call */

typedef struct {
  int32_t n_layers, d_model, n_heads, d_ff;
  int32_t vocab;                 /* rows of the token embedding table */
  int32_t logit_lo, logit_hi;    /* allowed id slice [lo, hi): only these ids get logits */
  int32_t grid_h, grid_w;        /* image token grid; G = grid_h * grid_w tokens per image */
  int32_t prefix_len;            /* P condition tokens in front of the image tokens */
  int32_t prefix_kind;           /* VVS_PREFIX_CLASS: ids into a class table whose last row (id
                                    n_classes) is the null class; VVS_PREFIX_DENSE: [P, d] vectors */
  int32_t n_classes;
  int32_t n_prompts;             /* B */
  int32_t max_nodes;             /* largest N of any verify call, <= VVS_MAX_T - 1 */
  int32_t dtype;                 /* VVS_FP32: fp32 weights, activations and KV cache;
                                    VVS_BF16: bf16 weights, GEMM/attention operands and KV cache,
                                    fp32 accumulation, fp32 residual stream and logits */
  float cfg_scale;               /* s in l_u + s (l_c - l_u) */
  float rms_eps;
  float rope_base;
  int32_t relax_k;               /* neighbours per id in the table given to vvs_set_neighbors */
  float relax_delta;             /* budget of target mass the relaxed rule may absorb */
  int32_t feature_slots;         /* token-level feature cache (Section 4.3): features kept per row,
                                    0 .. VVS_MAX_FEATURE_SLOTS (0 = none; the paper keeps 5) */
  int32_t feature_pre_norm;      /* 0: a feature is the input of the output head (after the final
                                    norm); 1: the residual stream in front of the final norm */
  int32_t draft_input;           /* 0: a target model (token embeddings are the inputs);
                                    1: a drafter context for vvs_draft: the input of a token is
                                    W_fc [embedding ; feature], and the weight list ends with one
                                    more tensor fc [2 d, d] */
  int32_t norm_mode;             /* bf16 contexts, where the output of an RMSNorm is rounded to bf16:
                                    VVS_NORM_AUTO: the library chooses per call - separate
                                      normalisation kernels (below), or, where that is faster, the
                                      fused layer: the operand of the projection behind a norm is
                                      bf16(x g) and the row factor rsqrt(mean x^2 + eps) multiplies the
                                      fp32 result of the projection (equal in exact arithmetic, a
                                      different rounding of the same operand);
                                    VVS_NORM_SEPARATE: always separate normalisation kernels, which
                                      round bf16(x * rsqrt(mean x^2 + eps) * g), the definition's own
                                      rounding point (more launches per layer) */
} vvs_config;
enum { VVS_NORM_AUTO = 0, VVS_NORM_SEPARATE = 1 };
#define VVS_MAX_FEATURE_SLOTS 8

/* Sizes in bytes of the three device buffers a context needs.  VVS_ESIZE if the shape is not
 * supported (bf16 needs d_model % 64 == 0, d_ff % 64 == 0, V_eff % 64 == 0, head size 64 or 128;
 * any dtype needs head size % 4 == 0, max_nodes < VVS_MAX_T). */
vvs_status vvs_query_sizes(const vvs_config* cfg, size_t* kv_bytes, size_t* workspace_bytes,
                           size_t* packed_weight_bytes);

/* Creates a context over caller-allocated device buffers (256-byte aligned).  Synchronous. */
vvs_status vvs_create(const vvs_config* cfg, void* d_kv, void* d_workspace, void* d_packed_weights,
                      vvs_ctx** out);
void vvs_destroy(vvs_ctx* ctx);
const char* vvs_last_error(const vvs_ctx* ctx);   /* ctx may be NULL: error of the last failed create/query */

/* Number of canonical weight tensors (2 + 9 * n_layers + 2, one more for a drafter context) in
 * this order:
 *   embed [vocab, d]; prefix_embed [n_classes + 1, d] (may be NULL for dense prefixes);
 *   per layer: g1 [d], wq [d,d], wk [d,d], wv [d,d], wo [d,d], g2 [d], wg [d,F], wu [d,F], wd [F,d];
 *   gf [d]; wout [d, vocab]; drafter contexts only: fc [2d, d] (rows 0..d-1 multiply the token
 *   embedding, rows d..2d-1 the feature).
 * Matrices are row-major [in, out] (activations multiply from the left); element type = dtype. */
int32_t vvs_num_weight_tensors(const vvs_config* cfg);

/* Repacks the canonical tensors (device pointers, host array of n pointers) into d_packed_weights.
 * The canonical tensors may be freed once the stream has passed this point. */
vvs_status vvs_load_weights(vvs_ctx* ctx, const void* const* d_tensors, int32_t n, vvs_stream s);

/* Neighbour table for the relaxed rule: int32 [vocab, relax_k] on the device, for every id its
 * nearest other ids in latent space in ascending distance.  Kept by reference. */
vvs_status vvs_set_neighbors(vvs_ctx* ctx, const int32_t* d_nbr);

/* Host-only check of a draft topology, with the same rules as vvs_verify (either array may be NULL;
 * both NULL = chain).  Outputs (host, may be NULL): h_depth int32 [T], h_parent_out int32 [N]. */
vvs_status vvs_check_tree(int32_t n_nodes, const int32_t* h_parent, const uint8_t* h_tree_mask, int32_t* h_depth,
                          int32_t* h_parent_out);

/* Prefill (Algorithm 2 of the supplementary material, first line): runs the P prefix tokens and then
 * n_forced teacher-forced image tokens of every row through the model under a causal mask, caches
 * their K/V, and samples the next image token of each prompt from the CFG-mixed distribution at
 * the last position by inverse CDF with d_uniform[b].  Resets the context state.
 *   d_prefix_cond  : class kind: int32 [B, P] class ids;      dense kind: dtype [B, P, d]
 *   d_prefix_uncond: class kind: int32 [B, P] or NULL (null class); dense kind: dtype [P, d], shared
 *   d_forced_tokens: int32 [B, n_forced] or NULL when n_forced == 0; n_forced <= G - 1
 *   d_uniform      : float [B] in [0, 1)
 *   d_first_token  : int32 [B] out (full-vocabulary id); it becomes the pending token. */
vvs_status vvs_prefill(vvs_ctx* ctx, const void* d_prefix_cond, const void* d_prefix_uncond,
                       int32_t n_forced, const int32_t* d_forced_tokens, const float* d_uniform,
                       int32_t* d_first_token, vvs_stream s);

/* One verification pass (Section 2; Algorithm 2: "logits <- M_T(C_t); a <- Verify(logits, C_t)").
 *   n_nodes      : N >= 0 (0 = plain AR sampling of one token)
 *   h_parent     : host int32 [N], h_parent[j-1] in [0, j-1] = parent of node j; NULL = chain
 *   h_tree_mask  : host uint8 [T, T], entry (i, j) != 0 iff j is i or an ancestor of i; may be NULL.
 *                  When both are given they must describe the same tree; when only the mask is
 *                  given the parents are derived from it.
 *   d_draft_tokens: int32 [B, N], full-vocabulary ids inside [logit_lo, logit_hi); siblings distinct
 *   d_draft_probs : float [B, T, V_eff]; row j = the distribution the children of node j were drawn
 *                   from (rows of leaves are not read)
 *   d_uniforms    : float [B, T, 2] in [0, 1): [b, c, 0] decides node c, [b, j, 1] draws the final
 *                   token when the walk ends at node j
 *   mode          : VVS_STRICT or VVS_RELAXED
 *   d_accept_len  : int32 [B] out, number of accepted draft tokens a_b
 *   d_path        : int32 [B, VVS_MAX_T] out, node ids of the accepted path: path[0] = 0, then a_b ids
 *   d_next_token  : int32 [B] out, resampled / bonus token (full-vocabulary id); -1 for a prompt whose
 *                   image is already complete (then a_b = 0)
 * Children of a node are tried in ascending node id; after a rejection the target becomes the
 * normalised positive part of (target - draft) and the rejected id leaves the draft distribution.
 * At most G - n_emitted_b - 1 draft tokens are accepted, so the final token still lies in the image.
 * The outcome is also kept in the workspace for vvs_kv_commit. */
vvs_status vvs_verify(vvs_ctx* ctx, int32_t n_nodes, const int32_t* h_parent, const uint8_t* h_tree_mask,
                      const int32_t* d_draft_tokens, const float* d_draft_probs, const float* d_uniforms,
                      int32_t mode, int32_t* d_accept_len, int32_t* d_path, int32_t* d_next_token,
                      vvs_stream s);

/* Verification with post verification (Section 4.1): the tokens that the previous, verification-free
 * step accepted without asking the target model ride in front of the new candidates and go through
 * the same pass.  They are nodes 1 .. n_post of the tree, a chain below the root (h_parent[j-1] = j-1
 * for j <= n_post), and every other node descends from node n_post; anything else is VVS_EINVAL.
 * They are accepted without a test (their d_draft_probs rows and d_uniforms entries are not read) and
 * count in accept_len / path; the end-of-image cap applies to them like to any accepted token.  The
 * pass gives them their K/V (committed by vvs_kv_commit like every accepted node), which restores
 * exact AR conditioning for the candidates behind them.  d_draft_tokens[b][0 .. n_post-1] are their
 * ids.  n_post = 0 is vvs_verify.  Everything else as in vvs_verify. */
vvs_status vvs_verify_post(vvs_ctx* ctx, int32_t n_nodes, int32_t n_post, const int32_t* h_parent,
                           const uint8_t* h_tree_mask, const int32_t* d_draft_tokens, const float* d_draft_probs,
                           const float* d_uniforms, int32_t mode, int32_t* d_accept_len, int32_t* d_path,
                           int32_t* d_next_token, vvs_stream s);

/* The acceptance stage alone (CFG mix, softmax, accept / resample, path walk) on logits supplied by
 * the caller: d_raw_logits float [R, T, V_eff] (row-major, row r = 2b + {0: conditional,
 * 1: unconditional}).  Same outputs as vvs_verify; does not touch the KV cache, and the outcome is
 * not available to vvs_kv_commit. */
vvs_status vvs_accept_from_logits(vvs_ctx* ctx, int32_t n_nodes, const int32_t* h_parent,
                                  const uint8_t* h_tree_mask, const float* d_raw_logits,
                                  const int32_t* d_draft_tokens, const float* d_draft_probs,
                                  const float* d_uniforms, int32_t mode, int32_t* d_accept_len,
                                  int32_t* d_path, int32_t* d_next_token, vvs_stream s);

/* vvs_accept_from_logits for callers that cannot allocate device memory and have no workspace to lend: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same result.
 * The stage's scratch (per-node partial results and per-node target distributions, which the other entry
 * points keep in the caller's workspace) lives in a static device array inside the library, of
 * VVS_NOALLOC_MAX_PROMPTS * VVS_MAX_T * 8 + VVS_NOALLOC_MAX_PROB_FLOATS * 4 bytes (about 16 MiB), held by every
 * GPU the library runs on until the process ends.  The call allocates and frees nothing.  VVS_ESIZE when
 * n_prompts > VVS_NOALLOC_MAX_PROMPTS, n_prompts * (n_nodes + 1) * V_eff > VVS_NOALLOC_MAX_PROB_FLOATS, or V_eff > 18432.
 * All calls on one GPU share that GPU's array: calls that overlap on one GPU (other streams, other contexts)
 * race; calls on one stream are safe.  The array keeps the last call's contents; nothing in it has to be cleared
 * (every entry a call reads is written by that call first).  Does not touch the KV cache, the workspace, or
 * the outcome kept for vvs_kv_commit; vvs_debug_logits does not see its distributions. */
#define VVS_NOALLOC_MAX_PROMPTS 64
#define VVS_NOALLOC_MAX_PROB_FLOATS (4 << 20)
vvs_status vvs_accept_from_logits_noalloc(vvs_ctx* ctx, int32_t n_nodes, const int32_t* h_parent,
                                          const uint8_t* h_tree_mask, const float* d_raw_logits,
                                          const int32_t* d_draft_tokens, const float* d_draft_probs,
                                          const float* d_uniforms, int32_t mode, int32_t* d_accept_len,
                                          int32_t* d_path, int32_t* d_next_token, vvs_stream s);

/* Section 4.1: moves the K/V of the pending token and of the accepted path of the last vvs_verify
 * into consecutive cache slots S_b .. S_b + a_b, advances S_b and n_emitted_b by a_b + 1 and makes
 * next_token the pending token.  Exactly one commit per verify. */
vvs_status vvs_kv_commit(vvs_ctx* ctx, vvs_stream s);

/* Token-level feature cache (Section 4.3; Algorithm 2, "UpdateCache").  vvs_prefill stores the feature
 * of the last prefilled position of every row, vvs_kv_commit appends the features of the tokens it
 * commits (pending token, then the accepted path, in order); a row keeps its feature_slots most
 * recent ones.  A feature is [d_model] values in the context's dtype rounding (bf16 contexts: bf16
 * values).  Reads them out oldest first:
 *   d_features float [R, feature_slots, d_model] out, row r: entries 0 .. count-1 valid, rest zero
 *   d_count    int32 [B] out, valid entries per row of prompt b (both of its rows hold the same number)
 * vvs_set_state does not touch the cache. */
vvs_status vvs_read_features(vvs_ctx* ctx, float* d_features, int32_t* d_count, vvs_stream s);

/* ---- The verification-free step (Sections 4.2 and 4.4).  Host-only helpers need no context. ----
 *
 * Candidate paths of a draft tree = its root-to-leaf node sequences (root excluded), ordered by the
 * node id of their leaf.
 *
 * vvs_select_unverified (Section 4.2, Eq. 1): draws one candidate path uniformly with the uniform
 * u in [0, 1) (path floor(u * |P|)) and keeps its first gamma = min(L_s, floor(mean path length))
 * nodes.  Topology arguments as in vvs_check_tree.  h_nodes: host int32 [VVS_MAX_T] out, the kept node
 * ids in path order (these are the tokens to hand to the next vvs_verify_post as its unverified
 * tokens); n_kept: their number (0 for an empty tree). */
vvs_status vvs_select_unverified(int32_t n_nodes, const int32_t* h_parent, const uint8_t* h_tree_mask, float u,
                                 int32_t* h_nodes, int32_t* n_kept);

/* Uniform-interval policy (Section 4.4): 1 iff step step_index (counted from 0) is verification-free for
 * interval i, i.e. (step_index + 1) % i == 0 with i >= 2; never two in a row. */
int32_t vvs_skip_uniform(int32_t step_index, int32_t interval);

/* Dynamic policy (Algorithm 1): 1 iff the last step was verified and similarity >= threshold. */
int32_t vvs_skip_dynamic(float similarity, float threshold, int32_t last_step_verified);

/* Latent codebook for vvs_path_similarity: float [vocab, dim] on the device, dim in [1, 64]; kept by
 * reference. */
vvs_status vvs_set_codebook(vvs_ctx* ctx, const float* d_embed, int32_t dim);

/* Weighted average similarity of the candidate paths (Eq. 2; Algorithm 1 "CompSim" after
 * "Downsample"): per prompt, S = sum_l w_l S_l with w_l proportional to alpha^l, where S_l is the mean
 * cosine similarity of the codebook embeddings of the tokens at position l over all unordered pairs of
 * the kept paths that reach position l.  Every stride-th path is kept, starting with the first.
 * Positions reached by fewer than two kept paths are left out (weights renormalised); with no such
 * position S = 1; an all-zero embedding has cosine 0.
 *   d_draft_tokens int32 [B, N] full-vocabulary ids (as for vvs_verify); d_similarity float [B] out.
 * Does not touch the model state; may run on another stream than a verify in flight. */
vvs_status vvs_path_similarity(vvs_ctx* ctx, int32_t n_nodes, const int32_t* h_parent, const uint8_t* h_tree_mask,
                               const int32_t* d_draft_tokens, float alpha, int32_t stride, float* d_similarity,
                               vvs_stream s);

/* One drafting call (Algorithm 2: "f_t <- Retrieve(C, a); C_t <- M_D(f_t, a)"; Section 3, "Stale
 * Feature Reusability"; Section 4.1): the drafter - a context created with draft_input = 1, one or more
 * decoder blocks of the target's kind, the same d_model, dtype, B, id slice, grid and kind of feature
 * (feature_pre_norm) as the target -
 * is conditioned on the n_ctx most recent features of the target's token-level feature cache paired,
 * by recency, with the n_ctx most recent tokens of the sequence, and fills a candidate tree of a fixed
 * shape level by level: node j >= 1 gets the input W_fc [embedding of its token ; feature the drafter
 * produced at its parent]; the distribution at a node is the softmax of the drafter's CFG-mixed logits
 * (the drafter context's cfg_scale); the c-th child of a node (ascending node id) carries the id with
 * the c-th largest mixed logit there, ties to the lower id.  The drafter keeps no state between calls:
 * a node attends to the n_ctx pairs, its ancestors and itself.  Pair i sits at image index
 * first + i with first = max(0, root - (n_ctx - 1)), root = emitted tokens of the target - 1 +
 * n_unverified; node j at first + n_ctx - 1 + depth(j).
 *   n_nodes, h_parent, h_tree_mask: the tree shape, as for vvs_verify (n_nodes >= 1)
 *   n_ctx          : 1 .. feature_slots of the target; every row of the target should hold that many
 *                    features (a missing feature is read as zeros); n_ctx + (number of nodes that have
 *                    children, root excluded) <= max_nodes + 1 of the drafter context
 *   d_recent_tokens: int32 [B, n_ctx] full-vocabulary ids, oldest first; the last one is the root (the
 *                    target's pending token, or the last token accepted without verification)
 *   n_unverified   : tokens accepted without verification since the target's last commit, 0 .. 8
 *                    (they move the root's position; their features do not exist: the cached ones
 *                    are paired with newer tokens - stale features)
 *   d_given_tokens : NULL, or int32 [B, N]: the nodes' tokens are taken from here (e.g. sampled by the
 *                    caller) and only the distributions are computed
 *   d_draft_tokens : int32 [B, N] out;  d_draft_probs: float [B, T, V_eff] out, row j = distribution of
 *                    the children of node j (zeros for a leaf): the layouts vvs_verify takes.
 * The target's state and feature cache are only read.  Same stream rules as every other call. */
vvs_status vvs_draft(vvs_ctx* drafter, vvs_ctx* target, int32_t n_nodes, const int32_t* h_parent,
                     const uint8_t* h_tree_mask, int32_t n_ctx, const int32_t* d_recent_tokens,
                     int32_t n_unverified, const int32_t* d_given_tokens, int32_t* d_draft_tokens,
                     float* d_draft_probs, vvs_stream s);

/* 1 if a forward over n_tokens query tokens per row (a verify call with n_tokens - 1 draft nodes, or a
 * prefill chunk) takes the fused layer described at vvs_config.norm_mode, 0 if it runs the separate
 * normalisation kernels.  Host only; ctx must not be NULL. */
int32_t vvs_plan_is_fused(const vvs_ctx* ctx, int32_t n_tokens);

/* Per-prompt state: int32 [3, B] out = cached length S_b, emitted image tokens, pending token. */
vvs_status vvs_read_state(vvs_ctx* ctx, int32_t* d_state, vvs_stream s);

/* Overwrites the per-prompt state with int32 [3, B] (same layout as vvs_read_state): rolls the context
 * back (or forward) to a cached length whose K/V are still in the cache, e.g. to replay one verify
 * call.  Cached slots below the given length must hold valid K/V; that is the caller's business.
 * Clears a pending (uncommitted) verify. */
vvs_status vvs_set_state(vvs_ctx* ctx, const int32_t* d_state, vvs_stream s);

/* Kernel-class timing for benchmarks.  While enabled, every kernel launch of prefill / verify /
 * commit is bracketed by HIP events recorded on the caller's stream (host objects; no device
 * memory).  vvs_timing_read waits for the recorded events and returns the number of launches and
 * their summed duration for one class since timing was enabled.  Where a layer's q/k/v projection and its
 * attention run as one launch (bf16, head size 64, up to 64 tokens per row), that launch counts as VVS_K_GEMM
 * and the attention class stays empty. */
enum { VVS_K_GEMM = 0, VVS_K_ATTENTION = 1, VVS_K_ACCEPT = 2, VVS_K_ELEMENTWISE = 3, VVS_K_COMMIT = 4, VVS_K_CLASSES = 5 };
vvs_status vvs_timing_enable(vvs_ctx* ctx, int32_t on);
vvs_status vvs_timing_read(vvs_ctx* ctx, int32_t kernel_class, int32_t* n_launches, float* total_ms);

/* Inspection of the last verify (or prefill, with T = 1; for a drafter context: the last level of the
 * last vvs_draft, T = its block tokens: the n_ctx pairs, then the nodes that have children ordered by
 * depth, then id): any pointer may be NULL.
 *   d_raw_logits float [R, T, V_eff]; d_mixed_logits float [B, T, V_eff]; d_probs float [B, T, V_eff]. */
vvs_status vvs_debug_logits(vvs_ctx* ctx, float* d_raw_logits, float* d_mixed_logits, float* d_probs,
                            vvs_stream s);

/* Cached K and V of one (layer, row) as float [n_slots, d_model] (head-major inside a row), slots
 * 0 .. n_slots - 1. */
vvs_status vvs_debug_kv(vvs_ctx* ctx, int32_t layer, int32_t row, int32_t n_slots, float* d_k, float* d_v,
                        vvs_stream s);

/* C[M, N] = A[M, K] * W[K, N] through the same repacking and GEMM kernels the forward uses (bf16
 * contexts: the MFMA path; n and k multiples of 64), for unit tests.  d_a dtype [M, K]; d_w dtype
 * [K, N] (canonical [in, out] layout); d_scratch of vvs_debug_gemm_scratch_bytes bytes, 256-byte
 * aligned; d_c float [M, N]. */
size_t vvs_debug_gemm_scratch_bytes(const vvs_ctx* ctx, int32_t m, int32_t n, int32_t k);
vvs_status vvs_debug_gemm(vvs_ctx* ctx, int32_t m, int32_t n, int32_t k, const void* d_a, const void* d_w,
                          void* d_scratch, float* d_c, vvs_stream s);

/* Plain device-to-device copy of `bytes` bytes (multiple of 16; 16-byte aligned pointers) with one
 * grid-stride kernel.  Reads and writes exactly `bytes`: used to calibrate hardware traffic counters. */
vvs_status vvs_debug_copy(vvs_ctx* ctx, void* d_dst, const void* d_src, size_t bytes, vvs_stream s);

/* Measures how fast a compute unit pulls bytes through its L1 - the figure that bounds the projection kernels of this
 * library.  Launches `n_workgroups` workgroups of `waves` waves (1..16); workgroup w reads the `region_bytes` (a multiple of
 * 8192) at d_src + w * wg_stride_bytes (16-byte aligned; stride 0: every workgroup reads the same region, which then stays
 * in L2 when it is small; the caller's buffer must hold (n_workgroups - 1) * wg_stride_bytes + region_bytes) `reps` times,
 * its waves taking 1 KiB blocks round-robin, 8 blocks in flight per wave.  mode 0: 16-byte loads into registers; mode 1: direct-to-LDS loads (the staging path of the
 * tiled GEMMs).  d_sink: uint32 [n_workgroups]; mode 0 leaves a checksum of what thread 0 of each workgroup read (the sum
 * over its loads of the xor of the four words), mode 1 leaves 0 - it only keeps the loads alive.  The caller times the launch;
 * bytes through the L1 of a CU = region_bytes * reps.  VVS_EINVAL for arguments out of these ranges. */
vvs_status vvs_debug_fill_probe(vvs_ctx* ctx, const void* d_src, size_t region_bytes, size_t wg_stride_bytes, int32_t reps, int32_t mode,
                                int32_t n_workgroups, int32_t waves, uint32_t* d_sink, vvs_stream s);

#ifdef __cplusplus
}
#endif
#endif /* VVS_H */
