/*
 * trispec.h — C ABI of the MI355X (gfx950) verification pass of TriSpec,
 * ternary speculative decoding with a lightweight proxy verifier.
 *
 * One call, trispec_verify(), runs what the paper calls Verify(M, X + [x_1..x_k]):
 * a single parallel forward of a decoder-only verifier (the proxy M_p, Sec. 3.2
 * Eq. 5, or the target M_t, Sec. 2.1 Eq. 2 / Sec. 3.2 Eq. 10) over a chain or
 * tree of drafted tokens against an existing KV cache, fused with the per-token
 * decision of Sec. 3.2: greedy acceptance s_i and tau_a (Eq. 6 greedy form,
 * Eq. 7), the top-1/top-2 margin predicate g and the trusted prefix tau_m
 * (Eq. 8, Eq. 9), and the routing into Case I (proxy finishes the round) or
 * Case II (escalate to the target).
 *
 * Conventions
 *  - Plain C.  Every call returns 0 (TRISPEC_OK) or a negative TRISPEC_E* code;
 *    nothing throws or aborts across this boundary.
 *  - "device" pointers are HIP device memory owned by the caller; "host" pointers
 *    are ordinary host memory.  The library owns only small host descriptors.
 *  - trispec_verify() / trispec_decide() / trispec_sample_decide() / trispec_kv_commit()
 *    allocate nothing, never synchronise with the host, and enqueue all work on the
 *    caller's stream; results land in caller-owned device buffers when the stream
 *    reaches them.
 *  - Matrices are row-major [out, in] (y = x W^T), dtype per trispec_model_config.
 *  - Node order: node 0 is the root (the last committed token, whose KV is not in
 *    the cache yet); parents[i] < i; M = n_nodes <= TRISPEC_MAX_NODES per sequence.
 */
#ifndef TRISPEC_H
#define TRISPEC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define TRISPEC_MAX_NODES 128  /* nodes per sequence (ancestor mask = two 64-bit words); the paper's trees hold 60.
                                  The sampling form (trispec_sample_decide*) takes chains of up to 64 nodes */
#define TRISPEC_MAX_BATCH 8
#define TRISPEC_MAX_ROWS 256   /* batch * n_nodes */

enum {
  TRISPEC_OK = 0,
  TRISPEC_ENULL = -1,        /* a required pointer is NULL */
  TRISPEC_ESHAPE = -2,       /* model shape not supported by the kernels */
  TRISPEC_ENODES = -3,       /* n_nodes / batch out of range */
  TRISPEC_ETREE = -4,        /* parents[] is not a topologically ordered tree */
  TRISPEC_EFORCED = -5,      /* n_forced out of range or forced nodes are not a chain */
  TRISPEC_ECAPACITY = -6,    /* ctx_len + n_nodes exceeds the cache capacity */
  TRISPEC_EWORKSPACE = -7,   /* workspace missing, misaligned or too small */
  TRISPEC_EARG = -8,         /* any other invalid argument (criterion, threshold NaN, ...) */
  TRISPEC_EMISMATCH = -9,    /* kv cache was created for another model / batch */
  TRISPEC_ELAUNCH = -10,     /* the HIP runtime refused a launch (hipGetLastError) */
  TRISPEC_ESTATE = -11       /* trispec_verify on a bf16 model before trispec_model_pack */
};

enum { TRISPEC_F32 = 0, TRISPEC_BF16 = 1 };

/* Trust predicate g (Sec. 3.2 Eq. 8; alternatives in Sec. 4.3 "Routing Criteria"). */
enum {
  TRISPEC_CRIT_MARGIN = 0,   /* g = 1{ top1(p) - top2(p) >= threshold }  (the paper's default) */
  TRISPEC_CRIT_TOP1 = 1,     /* g = 1{ top1(p) >= threshold }            (max-softmax confidence) */
  TRISPEC_CRIT_ENTROPY = 2   /* g = 1{ H(p) <= threshold }, H = -sum p ln p in nats.  Sec. 4.3 names an entropy
                                criterion among the routing rules it compares but only cites its definition;
                                this is the plain Shannon entropy of the verifier's distribution */
};

typedef struct {             /* plain data, copied by trispec_model_create */
  int32_t n_layers, hidden, n_q_heads, n_kv_heads, head_dim, ffn, vocab;
  int32_t dtype;             /* TRISPEC_F32 | TRISPEC_BF16: what the model STORES (weights, KV cache).
                                bf16 models round nothing else: activations reach the matrix cores
                                as bf16 high + low pairs (~16 bits), accumulation is fp32 */
  float rms_eps;
  float rope_base;
  int32_t qk_norm;           /* 1: queries and keys pass through an RMSNorm over head_dim (weights q_norm /
                                k_norm, shared by the heads of a layer, eps = rms_eps) before the rotary
                                embedding, as in the Qwen3 family the paper evaluates on; 0: no such norm */
} trispec_model_config;

typedef struct {             /* device pointers into caller-owned memory */
  const void *embed;         /* [vocab, hidden] */
  const void *lm_head;       /* [vocab, hidden] (may alias embed) */
  const void *final_norm;    /* [hidden] */
  /* host arrays of n_layers device pointers each: */
  const void *const *wq;     /* [n_q_heads*head_dim, hidden] */
  const void *const *wk;     /* [n_kv_heads*head_dim, hidden] */
  const void *const *wv;     /* [n_kv_heads*head_dim, hidden] */
  const void *const *wo;     /* [hidden, n_q_heads*head_dim] */
  const void *const *w_gate; /* [ffn, hidden] */
  const void *const *w_up;   /* [ffn, hidden] */
  const void *const *w_down; /* [hidden, ffn] */
  const void *const *norm_attn; /* [hidden] */
  const void *const *norm_ffn;  /* [hidden] */
  const void *const *q_norm;    /* [head_dim]; read only when qk_norm = 1 (may be NULL otherwise) */
  const void *const *k_norm;    /* [head_dim] */
} trispec_weights;

typedef struct trispec_model trispec_model;
typedef struct trispec_kv trispec_kv;
typedef struct trispec_timer trispec_timer;

/*
 * The verifier M_p or M_t (Sec. 3 intro): a pre-norm decoder with RMSNorm, rotary
 * position embedding (rotate-half pairing (j, j + head_dim/2), angle
 * position * rope_base^(-2j/head_dim)), grouped-query attention and a SwiGLU FFN.
 * Copies the config and the pointer tables (not the weights); the weights must
 * outlive the model.  Makes no HIP call.
 * Supported: head_dim in {64, 128}; n_q_heads a multiple of n_kv_heads;
 * bf16 additionally needs hidden, ffn and n_q_heads*head_dim multiples of 64,
 * n_kv_heads*head_dim a multiple of 32 and at most 8 query heads per kv head.
 * Errors: TRISPEC_ENULL, TRISPEC_ESHAPE.
 */
int trispec_model_create(const trispec_model_config *cfg, const trispec_weights *w,
                         trispec_model **out);
int trispec_model_destroy(trispec_model *m);

/*
 * bf16 models: one-time repack of the projection, FFN and LM-head matrices into the layout the
 * weight-streaming kernels read (per 32 output rows and 64 reduction elements, one contiguous
 * 4 KB block holding the matrix-core operand fragments in lane order, zero-padded rows), so that
 * every load instruction of the hot path reads 1 KB contiguous.  `packed_dev` is a caller-owned,
 * 256-byte aligned device buffer of trispec_model_pack_bytes() bytes that must outlive the model;
 * the repack kernels are enqueued on `stream` (NULL = default stream).  Once that work has
 * completed the hot path no longer reads wq..w_down and lm_head (the caller may release them);
 * embed and the norm vectors are still read in place.  fp32 models: pack_bytes is 0 and pack
 * is a no-op.  Required before trispec_verify on a bf16 model (TRISPEC_ESTATE otherwise).
 * Errors: TRISPEC_ENULL, TRISPEC_EARG (alignment), TRISPEC_ELAUNCH.
 */
int trispec_model_pack_bytes(const trispec_model *m, size_t *bytes);
int trispec_model_pack(trispec_model *m, void *packed_dev, void *stream);

/*
 * KV cache of the prefix X (Sec. 2.1: the pass conditions on X).  Caller-owned
 * device buffers, both of trispec_kv_bytes() bytes, dtype of the model:
 *   K: [n_layers][batch][n_kv_heads][capacity][head_dim]   keys after rotary embedding
 *   V: [n_layers][batch][n_kv_heads][head_dim][capacity]   values, TRANSPOSED
 *      (position-contiguous, so the P.V product reads matrix-core operands directly)
 * capacity must be a multiple of 64.  ctx_len[b] (host, [batch]) = tokens already cached.
 * trispec_verify writes the draft nodes' K/V into slots [ctx_len, ctx_len + n_nodes)
 * and does not advance ctx_len, so a verify call is repeatable.
 * Errors: TRISPEC_ENULL, TRISPEC_ENODES (batch), TRISPEC_ECAPACITY.
 */
int trispec_kv_bytes(const trispec_model *m, int32_t batch, int32_t capacity, size_t *bytes);
int trispec_kv_create(const trispec_model *m, void *k_dev, void *v_dev, int32_t batch,
                      int32_t capacity, trispec_kv **out);
int trispec_kv_set_len(trispec_kv *kv, const int32_t *ctx_len_host);
int trispec_kv_destroy(trispec_kv *kv);

/* Repack of ONE row-major bf16 matrix [n_rows, k] (k a multiple of 64) into the streaming layout of
 * trispec_model_pack — for matrices that are not part of a model, i.e. the adapter of
 * trispec_verify_opts.  `packed_dev`: 256-byte aligned, trispec_pack_matrix_bytes() bytes.
 * Errors: TRISPEC_ENULL, TRISPEC_EARG (sizes, alignment), TRISPEC_ELAUNCH. */
int trispec_pack_matrix_bytes(int32_t n_rows, int32_t k, size_t *bytes);
int trispec_pack_matrix(const void *w_dev, int32_t n_rows, int32_t k, void *packed_dev, void *stream);

/* Makes a verified path part of the context (Sec. 2.1 / Alg. 1: after a round the accepted
 * prefix is appended to the sequence; the token the verifier adds on top becomes the root of
 * the next round and is not cached yet).  For every sequence b the K/V rows that the last
 * trispec_verify wrote at slots ctx_len[b] + nodes[b][i], i < n_commit[b], are moved to slots
 * ctx_len[b] + i in every layer, and ctx_len[b] grows by n_commit[b] (on return, on the host;
 * the move itself is queued on `stream`, so later calls on that stream see it).
 *   nodes_host     HOST [batch][TRISPEC_PATH_STRIDE]: node ids in path order, strictly
 *                  increasing (root first: the forced chain, then the approved drafts — the
 *                  `path` output of trispec_verify, preceded by nodes 0..n_forced-2)
 *   n_commit_host  HOST [batch]: 0 .. TRISPEC_MAX_NODES
 * Errors: TRISPEC_ENULL, TRISPEC_ENODES (count out of range), TRISPEC_ETREE (ids not strictly
 * increasing or not below TRISPEC_MAX_NODES), TRISPEC_ECAPACITY, TRISPEC_ELAUNCH.  On error
 * nothing is changed. */
int trispec_kv_commit(trispec_kv *kv, const int32_t *nodes_host, const int32_t *n_commit_host,
                      void *stream);

/*
 * Case II hand-over (Sec. 3.2 (ii), Eq. 10; Algorithm 1's target call): the input of the target
 * pass after the proxy approved path = [v_0 .. v_tau_m] of its draft tree.  Host integers only, no
 * GPU work.  The target has no KV for the approved tokens yet, so they stay in the input as a
 * forced chain; of the draft tree only the subtree below v_tau_m survives (the target conditions
 * on x_1..x_tau_m and verifies the rest); every other branch is dropped.  Tokens that earlier
 * rounds emitted without running the target (Case I rounds) and that the target therefore has not
 * cached either go in front as `prefix`, at positions prefix_pos0, prefix_pos0 + 1, ...
 *   tokens, parents, positions  HOST [n_nodes]: the proxy pass's tree (parents[0] = -1, parents[i] < i)
 *   path                        HOST [path_len]: node ids v_0 = 0 .. v_tau_m, each the parent of the next
 *                               (trispec_verify's `path` output, accepted_len + 1 entries)
 *   prefix_tokens               HOST [n_prefix] (may be NULL when n_prefix = 0)
 * Outputs, HOST arrays of TRISPEC_MAX_NODES entries each: the new tokens / parents / positions in
 * the order prefix, path, subtree (ascending old id); old_id = the proxy-tree node of every entry
 * (-1 for prefix entries); *out_n_nodes; *out_n_forced = n_prefix + path_len, the n_forced of the
 * target's trispec_verify call.
 * Errors: TRISPEC_ENULL, TRISPEC_ENODES (n_nodes out of range, or more than TRISPEC_MAX_NODES
 * entries result: ingest the prefix by plain passes first), TRISPEC_ETREE (parents not a
 * topologically ordered tree, or path not a root path), TRISPEC_EARG (negative counts).
 */
int trispec_prune_reroot(const int32_t *tokens, const int32_t *parents, const int32_t *positions,
                         int32_t n_nodes, const int32_t *path, int32_t path_len,
                         const int32_t *prefix_tokens, int32_t n_prefix, int32_t prefix_pos0,
                         int32_t *out_tokens, int32_t *out_parents, int32_t *out_positions,
                         int32_t *out_old_id, int32_t *out_n_nodes, int32_t *out_n_forced);

/*
 * The same cache in PAGES of TRISPEC_KV_PAGE slots, for callers that hand out cache memory in
 * blocks (a serving layer's block manager; not something the paper needs).  Two pools of
 * trispec_kv_paged_bytes(m, n_pages) bytes each, dtype of the model:
 *   K: [n_layers][n_pages][n_kv_heads][TRISPEC_KV_PAGE][head_dim]
 *   V: [n_layers][n_pages][n_kv_heads][head_dim][TRISPEC_KV_PAGE]     (transposed, as above)
 * and a page table page_table_dev, DEVICE int32 [batch][max_pages_per_seq]: slot s of sequence b is
 * slot s % TRISPEC_KV_PAGE of page page_table[b][s / TRISPEC_KV_PAGE].  The kernels read the table
 * when they run, so the caller may rewrite it between calls (in stream order); entries must lie in
 * [0, n_pages) and cover slots [0, ctx_len + n_nodes) of every sequence when a pass runs — they are
 * device data: an entry outside the pool is clamped into it (wrong results, no stray access).  Capacity = max_pages_per_seq * TRISPEC_KV_PAGE.  Every other
 * call takes such a cache like a contiguous one; results are identical.
 * Errors: TRISPEC_ENULL, TRISPEC_ENODES (batch), TRISPEC_ECAPACITY (page counts), TRISPEC_EARG (alignment).
 */
#define TRISPEC_KV_PAGE 256
int trispec_kv_paged_bytes(const trispec_model *m, int32_t n_pages, size_t *bytes);
int trispec_kv_create_paged(const trispec_model *m, void *k_pool_dev, void *v_pool_dev, const int32_t *page_table_dev,
                            int32_t batch, int32_t max_pages_per_seq, int32_t n_pages, trispec_kv **out);

/* The context lengths a cache object holds now (they grow with trispec_kv_commit).
 *   ctx_len_host  HOST [batch], written.   Errors: TRISPEC_ENULL. */
int trispec_kv_get_len(const trispec_kv *kv, int32_t *ctx_len_host);

/* Device scratch needed by trispec_verify for up to `batch` sequences of up to
 * `max_nodes` nodes (256-byte aligned buffer).  Errors: TRISPEC_ENULL, TRISPEC_ENODES. */
int trispec_workspace_bytes(const trispec_model *m, int32_t batch, int32_t max_nodes,
                            size_t *bytes);

typedef struct {
  int32_t criterion;         /* TRISPEC_CRIT_* */
  int32_t n_forced;          /* >= 1: nodes 0..n_forced-1 are a chain of already approved
                                tokens (Case II re-rooting, Eq. 10); the walk starts at
                                node n_forced-1 and forced nodes do not count as accepted */
  void *workspace;           /* device */
  size_t workspace_bytes;
  float *debug_logits;       /* optional device [batch, n_nodes, vocab] fp32; NULL on the hot path */
  void *stream;              /* hipStream_t; NULL = the default stream */
  trispec_timer *timer;      /* optional per-kernel timer (measurement only); NULL on the hot path */
  float *hidden_out;         /* optional device [batch, n_nodes, hidden] fp32: the verifier's feature at
                                every node — the final-norm output the LM head reads — which the
                                drafter is re-seeded with after the round (Sec. 3.2, "Drafter
                                selection and adapter training"); NULL = not exported */
  int32_t launch_mode;       /* TRISPEC_LAUNCH_PER_MATMUL (0, default) | TRISPEC_LAUNCH_PER_LAYER: how the pass
                                is cut into kernel launches (same arithmetic either way) */
  /* Features for the drafter (Sec. 3.2 "Drafter selection and adapter training"; all optional, off on
     the plain hot path).  The drafter is re-seeded after a round with the verifier's features at the
     verified nodes; when the verifier was the proxy they first pass through a one-layer adapter into
     the feature space the drafter expects. */
  const int32_t *feature_layers; /* HOST [n_feature_layers], ascending layer indices in [0, n_layers): */
  int32_t n_feature_layers;      /* 0 .. TRISPEC_MAX_FEATURE_LAYERS                                     */
  float *features_out;       /* device [n_feature_layers][batch, n_nodes, hidden] fp32: the residual stream after
                                those layers (low / middle / high features of a multi-layer drafter) */
  const void *adapter_w;     /* device: the adapter matrix [adapter_dim, hidden], y = f W^T + b on the final-norm
                                features f (what hidden_out exports).  bf16 models: the PACKED copy made by
                                trispec_pack_matrix; fp32 models: the row-major fp32 matrix.  The paper gives
                                neither shape nor non-linearity of its "one-layer MLP adapter": one affine map */
  const float *adapter_bias; /* device [adapter_dim] fp32, or NULL */
  int32_t adapter_dim;       /* a multiple of 4, >= 4 */
  float *adapter_out;        /* device [batch, n_nodes, adapter_dim] fp32 */
  const int32_t *draft_ranks; /* optional device [batch, n_nodes] from trispec_draft_ranks, see accept_top_k */
  int32_t accept_top_k;      /* 0 or 1: a draft token is accepted iff it equals the verifier's argmax (Eq. 6,
                                greedy form).  k > 1: the relaxed acceptance that the appendix "relaxed
                                verification" studies — accepted iff it is among the verifier's top-k candidates
                                at its parent node (draft_ranks[child] < k; lowest-numbered such child first);
                                the verifier's own token where the walk stops is still its argmax.  Needs
                                draft_ranks (TRISPEC_EARG otherwise) */
  uint64_t *stamps;          /* optional device [n_layers][16] (measurement only): 100 MHz wall-clock ticks of
                                one workgroup at the phase boundaries of each layer launch — [0] start, then
                                per matmul (O, gate+up, down, next QKV) [1+3p] past the barrier, [2+3p] end of
                                the weight stream, [3+3p] arrived at the next barrier; NULL on the hot path */
} trispec_verify_opts;

/* TRISPEC_LAUNCH_PER_MATMUL: one launch per matmul (the faster cut on MI355X as measured, hence
 * the default).  TRISPEC_LAUNCH_PER_LAYER: bf16 models of up to 128 rows (batch * n_nodes) whose
 * widths allow it run the O projection, gate + up, down projection and the next layer's QKV
 * projection of every layer as ONE launch of a grid that is resident all at once, with device-side
 * barriers between the four and the next matmul's first weights requested while the last
 * workgroups of a matmul finish; shapes it cannot take fall back to one launch per matmul.  The
 * barrier waits are bounded: should the grid ever not be resident at once, the pass still ends,
 * with bit 2 of the status word set and meaningless outputs. */
enum { TRISPEC_LAUNCH_PER_MATMUL = 0, TRISPEC_LAUNCH_PER_LAYER = 1 };

#define TRISPEC_PATH_STRIDE (TRISPEC_MAX_NODES)
#define TRISPEC_MAX_FEATURE_LAYERS 8

typedef struct {             /* device pointers, caller-owned; any may be NULL to skip it */
  int32_t *accepted_len;     /* [batch]  min(tau_a, tau_m): approved draft tokens (Eq. 7, Eq. 9) */
  int32_t *token;            /* [batch]  Case I: the verifier's own token x_{tau_a+1} (correction or
                                         bonus); Case II: -1 */
  int32_t *escalate;         /* [batch]  1 iff tau_a >= tau_m (Case II: hand over to the target) */
  int32_t *path;             /* [batch, TRISPEC_PATH_STRIDE] node ids v_0..v_len of the approved
                                         path, then -1 */
  int32_t *argmax;           /* [batch, n_nodes] verifier top-1 token at each node */
  float *confidence;         /* [batch, n_nodes] top-1 softmax probability */
  float *margin;             /* [batch, n_nodes] top-1 minus top-2 probability (Eq. 8) */
  float *entropy;            /* [batch, n_nodes] Shannon entropy of the verifier's distribution at each node, nats
                                         (written by trispec_verify / trispec_decide only) */
  int32_t *status;           /* [1] device-side error bits: 1 = a draft token id outside [0, vocab);
                                         4 = a device-side barrier wait expired (results are not valid) */
} trispec_verify_out;

/*
 * One verification pass + decision (Sec. 3.2; Algorithm 1 "Verify" and the routing
 * that follows it).
 *   draft_tokens  device [batch, n_nodes]  token of each node (node 0 = root)
 *   tree_parents  host   [batch, n_nodes]  parents[0] = -1, 0 <= parents[i] < i
 *   positions     device [batch, n_nodes]  absolute rotary position (ctx_len + depth)
 *   threshold     lambda of Eq. 8.  0 => every node trusted => never escalates =>
 *                 the standard greedy acceptance of a target pass.
 * Node i attends to cache slots [0, ctx_len) and to the draft nodes on its root
 * path (itself included).  The distribution p_{j+1} of the paper is the one emitted
 * at path node v_j; the walk tests g(p_{j+1}) BEFORE looking for the child that
 * matches argmax p_{j+1}, because tau_a = tau_m is Case II.  Duplicate sibling
 * tokens: lowest node id wins.  Equal top logits: lowest token id is the argmax and
 * the margin is 0.
 * Errors (all detected on the host before anything is enqueued): TRISPEC_ENULL,
 * TRISPEC_ENODES, TRISPEC_ETREE, TRISPEC_EFORCED, TRISPEC_ECAPACITY,
 * TRISPEC_EWORKSPACE, TRISPEC_EARG, TRISPEC_EMISMATCH; TRISPEC_ELAUNCH afterwards.
 */
int trispec_verify(trispec_model *m, trispec_kv *kv, const int32_t *draft_tokens,
                   const int32_t *tree_parents, const int32_t *positions, int32_t n_nodes,
                   float threshold, const trispec_verify_opts *opts,
                   const trispec_verify_out *out);

/*
 * Re-run only the decision (Eq. 7-9 and routing) from the per-node statistics the
 * last trispec_verify left in this workspace — threshold / criterion sweeps.
 * batch / n_nodes / workspace must be those of that verify call (the statistics are found
 * by offset); calling it on a workspace no verify has filled yields unspecified decisions.
 * draft_tokens and tree_parents are those of THIS call: the walk may run over other drafts than
 * the pass did (same number of nodes).  Same argument meaning and host-side errors as trispec_verify.
 */
int trispec_decide(trispec_model *m, int32_t batch, const int32_t *draft_tokens,
                   const int32_t *tree_parents, int32_t n_nodes, float threshold,
                   const trispec_verify_opts *opts, const trispec_verify_out *out);

/*
 * Sampling form of the decision (temperature > 0) for a draft CHAIN of n_nodes = k + 1 nodes
 * (node 0 = last committed token, node i = i-th draft token; parents are implied).
 * Sec. 2.1: draft token x_i is accepted with probability min(1, p_v,i(x_i) / p_d,i(x_i)); at the
 * first rejection the replacement is drawn from norm(max(0, p_v,i - p_d,i)).  Sec. 3.2 Eq. 6 is
 * the same Bernoulli variable for the proxy; tau_a, the trust predicate g and tau_m (Eq. 7 - 9)
 * and the routing into Case I / Case II are those of trispec_verify, with p_v = softmax(logits / T)
 * also inside g.  Algorithm 1 prints the token after the accepted prefix as a plain draw from the
 * verifier's distribution; TRISPEC_RESAMPLE_DIRECT does that, TRISPEC_RESAMPLE_RESIDUAL follows
 * Sec. 2.1 (the rule that keeps the verifier's output distribution).  When every draft token is
 * accepted both draw the bonus token from p_v at the last node.  A residual without mass (the
 * supplied draft row dominates the verifier's everywhere) falls back to the direct draw.
 * Tree-shaped drafts need a multi-candidate rule the paper does not define: not provided.
 *
 * A pure function of its inputs; no model or cache is involved, no random numbers are drawn here:
 *   logits        device [batch, n_nodes, vocab] fp32: the pass's logits (trispec_verify's
 *                 debug_logits buffer)
 *   draft_tokens  device [batch, n_nodes]
 *   p_draft       device [batch, n_nodes - 1, vocab] fp32: row i is the drafter's distribution
 *                 from which node i + 1's token was drawn (may be NULL when n_nodes = 1)
 *   u_accept      device [batch, n_nodes] uniforms in [0, 1): entry i decides draft node i
 *                 (entries below n_forced are not read): accepted iff u * p_d(x) < p_v(x)
 *   u_sample      device [batch] uniforms in [0, 1): the token is the smallest v whose cumulative
 *                 mass (ascending token id) exceeds u * total mass
 *   scratch       device, 256-byte aligned, trispec_sample_scratch_bytes() bytes
 * out: accepted_len, token (-1 in Case II), escalate, path, argmax, confidence and margin (of the
 * tempered distribution), status (bit 0: a draft token id outside [0, vocab); such a token is
 * never accepted; bit 1: a draw found no usable mass — a logit, a draft probability or a uniform
 * that is NaN or infinite — and returned that node's argmax instead).  Any out pointer may be NULL.  Enqueues four kernels on `stream`, allocates
 * nothing, does not synchronise.
 * Errors (host side, before any launch): TRISPEC_ENULL, TRISPEC_ENODES (a chain of more than 64
 * nodes included), TRISPEC_EFORCED, TRISPEC_EWORKSPACE (scratch), TRISPEC_EARG (temperature not finite and positive, threshold NaN,
 * criterion, resample, vocab outside [1, 4194304]); TRISPEC_ELAUNCH afterwards.
 */
#define TRISPEC_RESAMPLE_RESIDUAL 0
#define TRISPEC_RESAMPLE_DIRECT 1

typedef struct {
  float temperature;         /* T > 0 */
  int32_t resample;          /* TRISPEC_RESAMPLE_* */
  int32_t criterion;         /* TRISPEC_CRIT_* */
  int32_t n_forced;          /* >= 1: nodes 0..n_forced-1 are already approved (Case II hand-over) */
  const float *p_draft;      /* device */
  const float *u_accept;     /* device */
  const float *u_sample;     /* device */
  void *scratch;             /* device */
  size_t scratch_bytes;
  void *stream;              /* hipStream_t; NULL = the default stream */
} trispec_sample_opts;

int trispec_sample_scratch_bytes(int32_t batch, int32_t n_nodes, int32_t vocab, size_t *bytes);
int trispec_sample_decide(const float *logits, const int32_t *draft_tokens, int32_t batch,
                          int32_t n_nodes, int32_t vocab, float threshold,
                          const trispec_sample_opts *opts, const trispec_verify_out *out);

/*
 * trispec_sample_decide for callers that cannot allocate device memory at all — code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc — and so cannot bring the
 * scratch buffer: the same four kernels run on a scratch area that is part of this library's
 * device image (TRISPEC_STATIC_SCRATCH_BYTES bytes per GPU, held until the process ends).
 * Arguments, outputs and host-side errors are those of trispec_sample_decide, except that
 * opts->scratch and opts->scratch_bytes are ignored; a (batch, n_nodes, vocab) whose
 * trispec_sample_scratch_bytes() exceeds TRISPEC_STATIC_SCRATCH_BYTES is refused with
 * TRISPEC_EWORKSPACE before anything is enqueued (batch 8 x 9 nodes x vocabulary 151936 needs
 * about 60 KB).  Call it with the GPU that owns opts->stream current.  It calls no hipMalloc /
 * hipFree and no allocating library routine; the first call on a GPU looks the area's address up
 * once (TRISPEC_ELAUNCH if that fails).  Every call on one GPU shares that GPU's area: calls that
 * overlap in time on one GPU (different streams, different threads) race and must be serialised
 * by the caller; calls in sequence need no clearing in between (no kernel reads an entry that the
 * same call has not written).
 */
#define TRISPEC_STATIC_SCRATCH_BYTES (1 << 20)
int trispec_sample_decide_static(const float *logits, const int32_t *draft_tokens, int32_t batch,
                                 int32_t n_nodes, int32_t vocab, float threshold,
                                 const trispec_sample_opts *opts, const trispec_verify_out *out);

/*
 * Measurement aid: HIP events recorded on the pass's own stream around every launch of one
 * kernel class, so a benchmark can price that kernel against the HBM roofline.
 *   TRISPEC_K_GEMM  the weight-streaming projection / FFN matmul (4 launches per layer)
 *   TRISPEC_K_HEAD  the fused LM-head + softmax-statistics kernel (1 launch per pass)
 *   TRISPEC_K_ATTN  the tree-masked attention of a layer (context kernel + merge kernel, one bracket)
 * create/destroy make HIP event calls (not for the hot path).  read() needs the stream to be
 * idle (caller synchronises); it returns the number of timed launches since the last reset,
 * their summed duration and the summed algorithmic HBM bytes of those launches (weights or
 * K/V read once).  Launches beyond `capacity` are not timed.
 * Errors: TRISPEC_ENULL, TRISPEC_EARG, TRISPEC_ELAUNCH (event call failed).
 */
enum { TRISPEC_K_GEMM = 0, TRISPEC_K_HEAD = 1, TRISPEC_K_ATTN = 2 };
int trispec_timer_create(int32_t kernel_class, int32_t capacity, trispec_timer **out);
int trispec_timer_reset(trispec_timer *t);
int trispec_timer_read(trispec_timer *t, int32_t *n_launches, double *total_ms, double *total_bytes);
int trispec_timer_destroy(trispec_timer *t);

/*
 * One sequence decoded by the ternary scheme, greedy form on draft trees (Algorithm 1; Sec. 3.2
 * Cases I and II, Eq. 10): the routing between proxy and target and the bookkeeping of the two
 * caches, as host code on top of trispec_verify, trispec_prune_reroot and trispec_kv_commit.
 * A round: the proxy verifies the draft tree at threshold lambda.  Case I (no escalation): the
 * approved path is committed to the proxy's cache and the proxy's own token ends the round; the
 * target does not run.  Case II: the target verifies, at threshold 0, the forced chain [tokens it
 * has not cached yet] + [approved path v_0..v_tau_m] plus the subtree under v_tau_m; both caches
 * commit what it accepted and its token ends the round.  The target's cache lags while rounds end
 * at the proxy; when lagging tokens and tree do not fit one pass of max_nodes nodes, plain passes
 * of the target ingest them first.
 * Unlike the calls above these BLOCK: routing is a host decision, so every pass is followed by a
 * copy of its decision to the host and a stream synchronisation.  They allocate no device memory.
 * The drafter is the caller's: every round brings its own tree.
 */
typedef struct trispec_ternary trispec_ternary;
#define TRISPEC_TERNARY_SCRATCH_INTS 1024
typedef struct {
  trispec_model *proxy, *target;              /* M_p and M_t; the same vocabulary */
  trispec_kv *kv_proxy, *kv_target;           /* caches of ONE sequence (batch 1), one per model */
  void *workspace_proxy, *workspace_target;   /* device; trispec_workspace_bytes(model, 1, max_nodes) each */
  size_t workspace_proxy_bytes, workspace_target_bytes;
  int32_t *scratch_dev;                       /* device, TRISPEC_TERNARY_SCRATCH_INTS int32 */
  int32_t criterion;                          /* TRISPEC_CRIT_* of the proxy pass (the target pass trusts itself) */
  int32_t max_nodes;                          /* 1 .. TRISPEC_MAX_NODES: the largest pass */
  void *stream;                               /* hipStream_t; NULL = the default stream */
} trispec_ternary_config;

typedef struct {                              /* decision of one pass, on the host */
  int32_t accepted_len, token, escalate, status, path_len;
  int32_t path[TRISPEC_PATH_STRIDE];
} trispec_pass_result;

typedef struct {
  int32_t escalate;                           /* 1 = Case II: the target ran */
  int32_t catch_up;                           /* plain target passes that first ingested lagging tokens */
  int32_t target_nodes, n_forced_target;      /* shape of the target's pass (Case II) */
  int32_t n_emitted;                          /* tokens this round appended to the sequence */
  int32_t ctx_len_proxy, ctx_len_target;      /* after the round */
  trispec_pass_result proxy, target;          /* `target` is meaningful in Case II only; its path is in
                                                 node ids of the target's (pruned, re-rooted) pass */
} trispec_round_info;

/* Copies the config; the objects it names must outlive the decoder.  Makes no HIP call.
 * Errors: TRISPEC_ENULL, TRISPEC_ENODES (max_nodes, cache batch != 1), TRISPEC_EMISMATCH (a cache of
 * another model, different vocabularies), TRISPEC_EARG (criterion), TRISPEC_EWORKSPACE. */
int trispec_ternary_create(const trispec_ternary_config *cfg, trispec_ternary **out);
int trispec_ternary_destroy(trispec_ternary *t);
/* New sequence: both caches are emptied and take in prompt[0 .. n_prompt-2] by plain passes; the
 * last prompt token is the first root.  prompt_host: HOST [n_prompt], n_prompt >= 1.
 * Errors: those of trispec_verify / trispec_kv_commit, TRISPEC_EARG (token ids, n_prompt). */
int trispec_ternary_start(trispec_ternary *t, const int32_t *prompt_host, int32_t n_prompt);
/* Takes over a sequence whose caches the caller has advanced by other means (e.g. rounds of the
 * sampling form): seq_host HOST [n_seq] is the emitted sequence; the proxy's cache must hold
 * n_seq - 1 tokens and the target's at most that.  Errors: TRISPEC_ENULL, TRISPEC_EARG. */
int trispec_ternary_resume(trispec_ternary *t, const int32_t *seq_host, int32_t n_seq);
/* One round.  parents_host / tokens_host: HOST [n_nodes], the draft tree (tokens_host[0] is ignored:
 * the root is the last token of the sequence); positions follow from the proxy cache's length and
 * the depths.  info_host (optional) receives what happened.  On an error from a pass nothing has
 * been committed by the failing step, but earlier steps of the round (catch-up passes) stay.
 * Errors: those of trispec_verify / trispec_prune_reroot / trispec_kv_commit, TRISPEC_EARG (a token id
 * outside the vocabulary, or a device-side status bit after a pass), TRISPEC_ESTATE (no sequence started). */
int trispec_ternary_round(trispec_ternary *t, const int32_t *parents_host, const int32_t *tokens_host,
                          int32_t n_nodes, float lambda, trispec_round_info *info_host);
/*
 * One round of the sampling form (temperature > 0) on a draft CHAIN tokens_host[0 .. n_nodes-1]
 * (tokens_host[0] is ignored: the root is the last token of the sequence), Algorithm 1 as printed:
 * the proxy accepts draft tokens by the Bernoulli rule of Eq. 6 and routes by Eq. 8 / 9 on its
 * tempered distribution (trispec_sample_decide on the pass's logits); in Case II the target verifies
 * the whole chain behind the tokens it has not cached yet, with x_1 .. x_tau_m taken as approved,
 * and its draw ends the round.  No random numbers are drawn here: the uniforms are the caller's.
 *   p_draft_dev           device [n_nodes - 1, vocab] fp32: row i = the drafter's distribution from
 *                         which draft token i + 1 was drawn (may be NULL when n_nodes = 1)
 *   u_accept_*_host       HOST [n_nodes] uniforms in [0, 1): entry i decides draft token i in the
 *                         proxy's / the target's pass; u_sample_*: the uniform of that pass's draw
 *   logits_dev            device work buffer [max_nodes, vocab] fp32 (the pass's logits)
 *   p_draft_work_dev      device work buffer [max_nodes - 1, vocab] fp32 (the draft rows shifted
 *                         behind the lagging tokens of the target's longer chain)
 * The decision kernels run on the library's own scratch area (trispec_sample_decide_static: calls
 * that overlap on one GPU race).  A chain — the draft chain, and the target's longer chain of lagging
 * tokens + draft chain — holds at most min(max_nodes, 64) nodes; a longer lag is taken in by plain
 * target passes first.  Errors: those of trispec_ternary_round and trispec_sample_decide.
 */
typedef struct {
  float temperature;                 /* T > 0 */
  int32_t resample;                  /* TRISPEC_RESAMPLE_* */
  const float *p_draft_dev;
  const float *u_accept_proxy_host, *u_accept_target_host;
  float u_sample_proxy, u_sample_target;
  float *logits_dev;
  float *p_draft_work_dev;
} trispec_sample_round;
int trispec_ternary_round_sample(trispec_ternary *t, const int32_t *tokens_host, int32_t n_nodes, float lambda,
                                 const trispec_sample_round *s, trispec_round_info *info_host);
/* View of the sequence emitted so far (prompt included), valid until the next call on `t`. */
int trispec_ternary_sequence(const trispec_ternary *t, const int32_t **tokens_host, int32_t *n_tokens);

/* Test hook: byte offset and size, inside the workspace of a verify call with these
 * (batch, n_nodes), of a named intermediate of the LAST layer ("x" residual stream fp32;
 * "attn_out" and "act", the O- and down-projection operands in the kernels' fragment order)
 * or of the per-node statistics behind the decision ("node_l1", "node_l2", "node_sum",
 * "node_idx").  Errors: TRISPEC_ENULL, TRISPEC_ENODES, TRISPEC_EARG (unknown name). */
int trispec_workspace_region(const trispec_model *m, int32_t batch, int32_t n_nodes,
                             const char *name, size_t *offset, size_t *bytes);

/*
 * Rank of every draft token under the verifier (appendix "relaxed verification", top-k
 * verification): ranks[b][i], i > 0, = the number of vocabulary entries that the verifier puts
 * before tokens[b][i] in the distribution emitted at node i's parent (larger logit, or equal
 * logit and lower token id); 0 = the parent's argmax; -1 for the root and for token ids outside
 * [0, vocab).  A pure function of materialised logits:
 *   logits        device [batch, n_nodes, vocab] fp32 (trispec_verify's debug_logits buffer)
 *   draft_tokens  device [batch, n_nodes];  tree_parents  HOST [batch, n_nodes]
 *   ranks         device [batch, n_nodes] int32, written when `stream` reaches the kernel
 * Feed it to trispec_decide through opts->draft_ranks with opts->accept_top_k = k.
 * Errors: TRISPEC_ENULL, TRISPEC_ENODES, TRISPEC_ETREE, TRISPEC_EARG (vocab < 1), TRISPEC_ELAUNCH.
 */
int trispec_draft_ranks(const float *logits, const int32_t *draft_tokens, const int32_t *tree_parents,
                        int32_t batch, int32_t n_nodes, int32_t vocab, int32_t *ranks, void *stream);

/* Test hooks of the bounded device-side wait.  trispec_debug_set_spin_limit: longest wait of any
 * later call, in ticks of the 100 MHz wall clock (0 restores the default of 2 s).
 * trispec_wait_probe: one workgroup waits on `counter_dev` (an int32 the caller leaves below
 * `expect`) exactly as a layer launch waits at a barrier — it must give up after limit_ticks, set
 * *abort_dev to 1 and OR 4 into *status_dev, and end normally; with *abort_dev already non-zero it
 * must not wait at all.  Errors: TRISPEC_ENULL, TRISPEC_ELAUNCH. */
int trispec_debug_set_spin_limit(uint64_t ticks);
int trispec_wait_probe(int32_t *counter_dev, int32_t expect, uint64_t limit_ticks, int32_t *abort_dev,
                       int32_t *status_dev, void *stream);

/* Algorithmic HBM bytes of one verify pass at this shape: layer weights once + LM head
 * once + context K/V once + draft K/V written (the figure the roofline is priced on). */
int trispec_pass_bytes(const trispec_model *m, int32_t batch, int32_t n_nodes,
                       const int32_t *ctx_len_host, double *bytes);

/* Plain device-to-device copy of `bytes` bytes (a multiple of 16; both pointers 16-byte
 * aligned, regions must not overlap) on `stream`, by one streaming kernel.  Not part of the
 * method: it is the measured streaming ceiling quoted next to the roofline, and the kernel of
 * known traffic (bytes read + bytes written) that memory counters are calibrated against.
 * Errors: TRISPEC_ENULL, TRISPEC_EARG (size or alignment), TRISPEC_ELAUNCH. */
int trispec_copy_probe(void *dst_dev, const void *src_dev, size_t bytes, void *stream);

const char *trispec_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* TRISPEC_H */
