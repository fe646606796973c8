/*
 * firp.h - C ABI of the MI355X-native FIRP decoding step.
 *
 * FIRP (Methodology / FIRP; Inference stage; Tree attention): in one forward pass of a
 * LLaMA-style decoder, k linear maps W_i h + b_i (Eq. 3) placed at an intermediate layer turn
 * the hidden state of a real token into k pseudo hidden states for the next k positions.  The
 * pseudo states, the real token and a tree of draft candidates run through the remaining
 * layers under a tree attention mask over the KV cache; the original lm-head verifies the
 * candidates greedily (longest accepted path) and drafts the next tree from the pseudo rows;
 * the accepted path is committed to the cache.  The returned tokens are exactly those of
 * sequential greedy decoding (Eq. 1).
 *
 * Conventions
 *  - Every call returns FIRP_OK or a negative firp_status; firp_last_error() gives text.
 *  - All argument and capacity checks run on the host before anything is enqueued; a failed
 *    call leaves the context unchanged.
 *  - The library never allocates or frees device memory and creates no streams: weights, the
 *    workspace and the stream are the caller's.  (Two exceptions, both stated where they
 *    apply: firp_debug_gemm_static owns one fixed buffer per GPU, and a step replayed as a
 *    captured graph - option "graph" - holds what the HIP runtime allocates for the graph.)  Pointers marked DEVICE must be device
 *    addresses valid on the current HIP device; pointers marked HOST are ordinary host memory
 *    read or written during the call only.
 *  - Weights are `[out, in]` row-major in `dtype`, borrowed: they must outlive the context
 *    and are never written.
 *  - One context, one thread.  Calls on one context are serialised by the caller.
 */
#ifndef FIRP_H
#define FIRP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct firp_ctx firp_ctx;

typedef enum {
  FIRP_OK = 0,
  FIRP_EINVAL = -1,    /* malformed argument (null, out of range, bad tree, bad dtype) */
  FIRP_ESTATE = -2,    /* call out of order (step before prefill) */
  FIRP_ECAPACITY = -3, /* exceeds max_ctx / max_nodes / max_rows / workspace */
  FIRP_EDEVICE = -4    /* a HIP call failed */
} firp_status;

typedef enum { FIRP_F32 = 0, FIRP_BF16 = 1 } firp_dtype;

#define FIRP_MAX_K 8      /* pseudo hidden states per anchor */
#define FIRP_MAX_B 16     /* candidates kept per future position (top-b) */
#define FIRP_MAX_ROWS 256 /* rows of one sequence in one step: N + k*|A| */

/* Shapes, numerics and capacities (the decoder of Experiment / Setup: LLaMA-2 style). */
typedef struct {
  int32_t n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab;
  float rms_eps, rope_base;
  int32_t dtype;     /* firp_dtype of weights and KV cache */
  int32_t max_ctx;   /* committed tokens the cache can hold, per sequence */
  int32_t max_batch; /* independent sequences */
  int32_t max_nodes; /* N, tree nodes including the root */
  int32_t max_rows;  /* N + k*|A| <= FIRP_MAX_ROWS; also the prefill chunk length */
  int32_t b_max;     /* top-b kept per pseudo row, 1..FIRP_MAX_B */
} firp_model_desc;

/* DEVICE pointers.  Per-layer entries are HOST arrays of n_layers DEVICE pointers. */
typedef struct {
  const void *embed;             /* [V, d] */
  const void *const *wq;         /* [Hq*dh, d] */
  const void *const *wk;         /* [Hkv*dh, d] */
  const void *const *wv;         /* [Hkv*dh, d] */
  const void *const *wo;         /* [d, Hq*dh] */
  const void *const *w_gate;     /* [F, d] */
  const void *const *w_up;       /* [F, d] */
  const void *const *w_down;     /* [d, F] */
  const void *const *norm_attn;  /* [d] */
  const void *const *norm_mlp;   /* [d] */
  const void *norm_final;        /* [d] */
  const void *lm_head;           /* [V, d] */
} firp_weights;

/*
 * Draft-tree topology (Tree attention: "a pre-defined tree structure and parser").
 * HOST arrays borrowed for the call.  Node 0 is the root: the last emitted token, which is
 * not yet in the cache.  Nodes are in topological order.  Node v at depth j >= 1 carries the
 * candidate drafts[j-1][rank[v]] produced by the previous step.  anchor[v] = 1 gives node v
 * k pseudo rows (Eq. 3 applied to its hidden state); the next tree can be drafted only if the
 * accepted path ends at an anchor, otherwise the next step runs on the root alone.
 */
typedef struct {
  int32_t n_nodes;        /* N >= 1 */
  const int32_t *parent;  /* parent[0] = -1, 0 <= parent[v] < v */
  const int32_t *rank;    /* 0 <= rank[v] < b_max; ignored for the root */
  const uint8_t *anchor;  /* NULL = every node is an anchor */
} firp_tree;

/* Bytes of DEVICE workspace firp_init needs for this description (0 on invalid input).
 * For a bf16 model this includes a second copy of every projection matrix (q, k, v, o, gate,
 * up, down, lm-head and the k maps: about the size of the model) in the fragment-major layout
 * the projection kernel streams; see firp_init. */
size_t firp_workspace_bytes(const firp_model_desc *desc, int32_t k);

/*
 * Create a context (FIRP: k maps at one intermediate layer).
 *  proj_w: HOST array of k DEVICE pointers, each [d, d]; proj_b: same for [d], or NULL.
 *  layer_l: the pseudo rows enter decoder layer `layer_l` (0-based): they are computed from
 *           the residual stream after layer_l layers and traverse n_layers - layer_l layers.
 *  workspace: DEVICE, >= firp_workspace_bytes, 256-byte aligned, owned by the caller and
 *           used exclusively by this context until firp_destroy.
 *  hip_stream: hipStream_t on which all work is enqueued (0 = the null stream).
 * firp_init itself touches no device memory.  For a bf16 model the first firp_prefill copies
 * the projection matrices into the workspace in the kernel's streaming layout (once, on the
 * stream); from then on the caller's q/k/v/o/gate/up/down/lm-head/proj_w buffers are read
 * only if the plain kernels are selected with firp_set_option("gemm", 0).  The embedding
 * table, the norm gains and the biases are always read in place.
 */
firp_status firp_init(firp_ctx **out, const firp_model_desc *desc, const firp_weights *weights,
                      const void *const *proj_w, const void *const *proj_b, int32_t layer_l,
                      int32_t k, void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * The same with one prediction layer per step (Training stage: "the index of prediction layer
 * for step i", t_i; Experiment / Setup uses three different layers for the three steps):
 *  layers: HOST array of k entries, 0 <= layers[0] <= ... <= layers[k-1] <= n_layers; pseudo
 *          hidden state i+1 of an anchor is W_i h + b_i of the anchor's residual stream entering
 *          decoder layer layers[i] and traverses the layers from there on, so the step carries
 *          N rows below layers[0] and N + (i+1) * anchors rows from layers[i] on.
 * firp_init(layer_l) is firp_init_layers with every entry equal to layer_l.
 */
firp_status firp_init_layers(firp_ctx **out, const firp_model_desc *desc, const firp_weights *weights,
                             const void *const *proj_w, const void *const *proj_b,
                             const int32_t *layers, int32_t k, void *workspace,
                             size_t workspace_bytes, void *hip_stream);

/*
 * Start `batch` sequences (Inference stage, first round): run the prompt through the decoder
 * to fill the cache, then a root-only step on the last prompt token.
 *  tokens: HOST, the prompts concatenated; lens: HOST [batch], each >= 1 and <= max_ctx.
 *  first_token: HOST [batch], receives the first generated token of each sequence.
 * Synchronises the stream before returning.
 */
firp_status firp_prefill(firp_ctx *ctx, int32_t batch, const int32_t *tokens,
                         const int32_t *lens, int32_t *first_token);

/*
 * One decoding step (Inference stage): verify the tree drafted by the previous step, emit
 * the accepted candidates plus one more token, draft the next tree, commit the path.
 *  accepted: HOST [batch][FIRP_MAX_K + 1]; row b receives n_accepted[b] tokens in order
 *            (the accepted candidates, then the token that follows them).
 *  n_accepted: HOST [batch], each in 1 .. (deepest level of `tree`) + 1.
 * The tree may be at most FIRP_MAX_K levels deep; levels beyond k receive no candidates from
 * the drafts (they can only be filled through firp_step_with_candidates).
 * Synchronises the stream before returning (the step's only synchronisation).
 */
firp_status firp_step(firp_ctx *ctx, const firp_tree *tree, int32_t *accepted,
                      int32_t *n_accepted);

/*
 * Forward pass of the Training stage for prediction step `step` (1..k) on one sequence of n
 * tokens (Training stage, Eq. 3-4), forward only: the n hidden states entering the step's
 * prediction layer are mapped to n pseudo hidden states and appended; pseudo row j (the stand-in
 * for position j + step) sees hidden states 1 .. j + step - 1 and itself and carries position id
 * j + step; all 2n rows pass the remaining layers and the lm-head.
 *   loss: HOST, receives sum_{q=1}^{n-step} KL(P~_q, P_{q+step}), KL(A,B) = sum_t A_t log(A_t/B_t);
 *   kl:   HOST [n - step] or NULL, the terms of the sum.
 * Needs a context that holds no sequence (fresh, or after firp_reset) and 2n <= max_rows; uses
 * sequence 0's cache slots as scratch and leaves the context without sequences.  The 2n rows
 * of logits can be read with firp_debug_last_logits afterwards.
 */
firp_status firp_train_forward(firp_ctx *ctx, const int32_t *tokens, int32_t n, int32_t step,
                               double *loss, float *kl);

/* Drop all sequences (the cache becomes empty); weights and workspace stay. */
firp_status firp_reset(firp_ctx *ctx);

/* Free host state.  The workspace and the weights remain the caller's. */
void firp_destroy(firp_ctx *ctx);

/* Text of the last error on this context (or of the last failed firp_init when ctx is NULL). */
const char *firp_last_error(const firp_ctx *ctx);

/* ---- test / debug surface (not on the hot path) ------------------------------------- */

/* As firp_step, but the candidates come from the caller: node_tokens HOST [batch][N],
 * entry 0 of each row ignored (the root is always the last emitted token). */
firp_status firp_step_with_candidates(firp_ctx *ctx, const firp_tree *tree,
                                      const int32_t *node_tokens, int32_t *accepted,
                                      int32_t *n_accepted);

/* Run only the host-side validation of a topology against this context's capacities (what
 * firp_step does first); n_rows (may be NULL) receives N + k*|A|.  Touches no device. */
firp_status firp_check_tree(firp_ctx *ctx, const firp_tree *tree, int32_t *n_rows);

/*
 * Draft-tree topology for a node budget (Experiment / Setup: the best tree structure is searched
 * for every budget of tree nodes).  accept: HOST [k][b] acceptance rates in [0, 1]: accept[i][r]
 * is the rate at which the rank-r candidate of prediction step i+1 is the target's token given
 * that its parent was accepted.  Under greedy verification a node is accepted with the product
 * of the rates along its path, and a step yields 1 + the sum of these products tokens on
 * average; the function returns the tree of at most n_nodes nodes (root included) that
 * maximises this (ties: shallower node first, then the smaller rank path), nodes in an order
 * firp_step accepts (parent before child).  parent / rank: HOST arrays of n_nodes entries;
 * n_out receives the node count (smaller than n_nodes when fewer nodes have a non-zero
 * product); expected_tokens (may be NULL) receives the objective.  Host only, no device work.
 */
firp_status firp_build_tree(const float *accept, int32_t k, int32_t b, int32_t n_nodes,
                            int32_t *parent, int32_t *rank, int32_t *n_out,
                            double *expected_tokens);

/* Logits of the last step, HOST [batch][T_hi][V] fp32, rows in step order: the tree nodes, then
 * pseudo row 1 of every anchor (ascending node id), then pseudo row 2 of every anchor, ...
 * n_rows receives T_hi.  A decoding step writes its logits to memory only with the option
 * "keep_logits" set (it needs no more than the greedy token of every node and the top-b ids of
 * every pseudo row); without it this call returns FIRP_ESTATE. */
firp_status firp_debug_last_logits(firp_ctx *ctx, float *logits, int32_t *n_rows);

/* Node ids of the last accepted path, HOST [batch][FIRP_MAX_K + 1]. */
firp_status firp_debug_last_path(firp_ctx *ctx, int32_t *path_nodes);

/* Current drafts, HOST [batch][k][b_max]; valid HOST [batch] (0 = next step is root-only).
 * drafts may be NULL: then only the flags are returned, from the host's mirror, with no device
 * work and no synchronisation. */
firp_status firp_get_drafts(const firp_ctx *ctx, int32_t *drafts, int32_t *valid);

/* Committed cache length of each sequence, HOST [batch]. */
firp_status firp_get_ctx_len(const firp_ctx *ctx, int32_t *len);

/* Copy the committed cache of one layer to the host as fp32: k_out, v_out HOST
 * [len][Hkv][dh] (len = committed length of sequence `seq`). */
firp_status firp_debug_read_cache(firp_ctx *ctx, int32_t seq, int32_t layer, float *k_out,
                                  float *v_out);

/* Behaviour switches for tests and measurements.  name = "gemm" value 0 (plain tiled kernel)
 * or 1 (MFMA weight-streaming kernel, bf16 models only; the default for them); "time_gemm" 0/1
 * (see firp_get_gemm_timing); "keep_logits" 0/1 (default 0: see firp_debug_last_logits);
 * "graph" 0 / 1 / 2: replay the decoding step of a resident topology as a captured HIP graph
 * never / whenever the stream and the kernels allow it / only for models whose step is short
 * enough for the replay to pay (the default; the stream must not be the legacy default stream).  Returns FIRP_EINVAL for an unknown name or value. */
firp_status firp_set_option(firp_ctx *ctx, const char *name, int32_t value);

/* With option "time_gemm" = 1 every launch of the MFMA projection kernel inside firp_step is
 * bracketed by HIP events on the library's stream; this returns the totals since the option
 * was set: kernel launches, their summed duration, and the weight bytes they streamed. */
firp_status firp_get_gemm_timing(const firp_ctx *ctx, int64_t *launches, double *total_ms,
                                 double *weight_bytes);

/* Counters of the context since firp_init, by name: "topo_uploads" = tree topologies whose
 * tables were uploaded to the device (the last few topologies stay resident: switching
 * between them, e.g. between a tree and its root-only sub-tree, uploads nothing).
 * FIRP_EINVAL for an unknown name. */
firp_status firp_get_stat(const firp_ctx *ctx, const char *name, int64_t *value);

/* What a pair of HIP events with nothing between them reads on the library's stream (mean over
 * the steps since "time_gemm" was set, one empty bracket per step; 0 before any): the share of
 * a bracketed launch's reading that is not the kernel. */
firp_status firp_get_event_overhead(const firp_ctx *ctx, double *bracket_ms);

/* Standalone entry to the projection kernel for per-kernel parity and bandwidth tests:
 * y[R, n] (DEVICE fp32) = x[R, K] (DEVICE fp32) . w[n, K]^T (DEVICE, `dtype`), on `hip_stream`,
 * using `workspace` (DEVICE, >= firp_gemm_workspace_bytes(R, n, K)) for operand planes,
 * split-K partial sums and (kind 1) the fragment-major copy of w, which every call remakes.  `kind` selects the kernel as the "gemm" option does. */
size_t firp_gemm_workspace_bytes(int32_t rows, int32_t n, int32_t k_dim);
firp_status firp_debug_gemm(const float *x, const void *w, float *y, int32_t rows, int32_t n,
                            int32_t k_dim, int32_t dtype, int32_t kind, void *workspace,
                            size_t workspace_bytes, void *hip_stream);

/* The same projection (firp_debug_gemm with bf16 w and kind 1) for callers that cannot
 * allocate device memory or pass a workspace: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  It calls no allocating routine.  Its scratch (operand
 * planes, partial sums, the fragment-major copy of w) is one fixed buffer of
 * firp_gemm_static_capacity() bytes (32 MiB) per GPU, held from the first use on that GPU until
 * the process ends; shapes whose firp_gemm_workspace_bytes(rows, n, k_dim) exceed it are
 * rejected with FIRP_ECAPACITY (firp_last_error(NULL) says by how much) before anything is
 * enqueued.  x, w (bf16 [n, K]), y are DEVICE pointers of the current device; the work is
 * enqueued on `hip_stream`.  Every call on a GPU uses that GPU's one buffer: calls that overlap
 * on one GPU (two streams, two threads) race; calls in stream order do not.  Nothing in the
 * buffer needs to start at zero: each call rewrites every byte it later reads. */
size_t firp_gemm_static_capacity(void);
firp_status firp_debug_gemm_static(const float *x, const void *w, float *y, int32_t rows, int32_t n,
                                   int32_t k_dim, void *hip_stream);

/* Measurement aid: one kernel that only reads `bytes` (>= 16, a multiple of 16 is read) of DEVICE
 * memory at `src` (16-byte aligned) on `hip_stream`; `sink` is 4 bytes of DEVICE memory it may
 * write.  Timing it over a buffer larger than every cache gives the streaming-read rate a kernel
 * can reach on this chip, which bench.py reports beside the step's bandwidth. */
firp_status firp_debug_stream_read(const void *src, size_t bytes, void *sink, void *hip_stream);

/* Host only: the launch plan the library picks for a projection of `rows` activation rows with an
 * [n, K] bf16 weight matrix (no device work; for tests of the planning logic).  Out (HOST, each may
 * be NULL): split-K factor, K elements per split (a multiple of 64), waves per workgroup (each owns
 * 32 rows of W), workgroups of one launch, and the activation rows one launch takes (128, or 256
 * when the kernel for 129..256 rows applies).  FIRP_EINVAL for a shape the MFMA kernels do not take
 * (rows < 1, n % 4 != 0, K % 8 != 0). */
firp_status firp_debug_gemm_plan(int32_t rows, int32_t n, int32_t k_dim, int32_t *splits, int32_t *k_per_split,
                                 int32_t *waves, int32_t *grid, int32_t *row_block);

#ifdef __cplusplus
}
#endif
#endif /* FIRP_H */
