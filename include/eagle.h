/*
 * libeagle -- one EAGLE speculative-decoding step on one AMD MI355X (gfx950), C ABI.
 *
 * The library implements the method of arXiv 2401.15077:
 *   drafting     (Sec. 3.1, App. A.1): the Autoregression Head -- concat(feature, embedding of the token one
 *                step ahead) -> FC 2d->d -> one decoder layer -> the target's LM head -- run once per tree
 *                level to expand a static draft tree; greedy children are the top-k tokens, non-greedy
 *                children are k tokens sampled without replacement;
 *   verification (Sec. 3.3): ONE target forward over all tree nodes with tree attention;
 *   acceptance   (Sec. 2 "Speculative sampling", App. A.2 Alg. 1): greedy walk, or multi-round speculative
 *                sampling applied recursively at every node; the accepted tokens' KV rows and features are
 *                kept for the next drafting phase (Sec. 3.3, last sentence).
 *
 * Conventions
 *   - Every call returns 0 (EAGLE_OK) or a negative error code; eagle_last_error() gives the text.
 *     Nothing throws or aborts across the boundary.
 *   - "dev" pointers are device (HIP) addresses, "host" pointers are ordinary host memory.
 *   - The library NEVER allocates device memory.  The caller hands in one workspace of
 *     eagle_workspace_bytes() bytes (256-byte aligned) that must stay valid until eagle_free();
 *     weights are copied (re-tiled) into that workspace by eagle_load_weight(), after which the caller may
 *     release its own copy.
 *   - All work is enqueued on the hipStream_t given to eagle_init().  Calls that return host data
 *     synchronise that stream; the others are asynchronous.
 *   - Sequences are slots 0..max_batch-1.  eagle_prefill() activates a slot; the step calls
 *     (draft / verify / accept / step / vanilla) act on ALL active slots at once, which must be slots
 *     0..n_active-1.  Calls on one context must not overlap in time.
 *   - Static draft tree: n_nodes nodes in BFS order, node 0 is the root (the last committed token, whose
 *     target forward has not run yet), parent[0] = -1, parent[v] < v, rank[v] = v's index among its
 *     siblings (0 = most probable).  At most 64 nodes.
 */
#ifndef EAGLE_H
#define EAGLE_H
#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct eagle_ctx eagle_ctx;

enum { EAGLE_OK = 0, EAGLE_EINVAL = -1, EAGLE_ENOMEM = -2, EAGLE_ESEQ_FULL = -3, EAGLE_ESTATE = -4, EAGLE_EHIP = -5 };
enum { EAGLE_F32 = 0, EAGLE_BF16 = 1 };

typedef struct {
  int32_t dtype;                      /* EAGLE_F32 | EAGLE_BF16: type of the weight matrices (and of the embedding) */
  int32_t kv_dtype;                   /* EAGLE_F32 | EAGLE_BF16: storage type of the KV cache entries */
  int32_t n_layers, d_model, n_heads, n_kv_heads, head_dim, d_ffn, vocab;
  int32_t n_experts, experts_per_tok; /* 0,0 = dense MLP; else top-k routed SwiGLU experts */
  int32_t draft_moe;                  /* the head's decoder layer is a MoE layer too */
  float rms_eps, rope_theta;
  int32_t max_batch, max_seq, page_tokens; /* KV paging: page_tokens slots per page (power of two) */
  int32_t n_nodes;                    /* draft tree (host arrays, copied) */
  const int32_t *parent, *rank;
  float temperature;                  /* 0 = greedy */
  uint64_t seed;                      /* counter-based generator for the non-greedy draws */
  int32_t weight_bits;                /* 0 or 16: weight matrices stay in `dtype`.  4: eagle_load_weight quantises every
                                         weight matrix of the layers, the head's FC and the LM head (not the embedding)
                                         to 4 bits as it copies it (Sec. 4.2: the int4 case study) -- weight-only,
                                         symmetric, per output row and group of 128 input columns: scale = bf16(max|w| / 7),
                                         code = clip(rint(w / scale), -8, 7), value scale * code.  Needs a dense bf16
                                         model whose widths are multiples of 128, and at most 32 rows per pass
                                         (max_batch * n_nodes <= 32); the prompt then runs 32 rows at a time. */
  int32_t head_loss_rows;             /* 0: off.  > 0: the workspace also holds what eagle_head_loss needs -- a second
                                         copy of the LM head re-tiled for the product with its transpose, and one
                                         pass's gradient of the logits -- (about 2 * vocab * d_model + 4 * vocab * pass
                                         rows bytes); needs a bf16 model with weight_bits 0 / 16 and vocab % 64 == 0.
                                         The value itself only switches the feature on: any row count is processed in
                                         passes. */
} eagle_config;

/* Which tensor eagle_load_weight() is given.  Matrices are row-major [out_features, in_features] in the
 * model dtype; norm gains and the FC bias are fp32 vectors.  MoE expert matrices are [n_experts, out, in]; the
 * router is an [n_experts, d_model] matrix in the model dtype (the library keeps and applies it in fp32). */
enum {
  EAGLE_W_EMBED = 0, EAGLE_W_LM_HEAD, EAGLE_W_FINAL_NORM, EAGLE_W_FC, EAGLE_W_FC_BIAS,
  EAGLE_W_ATTN_NORM, EAGLE_W_Q, EAGLE_W_K, EAGLE_W_V, EAGLE_W_O, EAGLE_W_MLP_NORM, EAGLE_W_ROUTER,
  EAGLE_W_GATE, EAGLE_W_UP, EAGLE_W_DOWN, EAGLE_W_COUNT
};
#define EAGLE_HEAD_LAYER (-1)         /* `layer` argument naming the Autoregression Head's decoder layer */

/* Device bytes the context needs for this config (weights in library layout, KV pages, activations). */
size_t eagle_workspace_bytes(const eagle_config *cfg);

/* Create a context inside `workspace_dev` (size >= eagle_workspace_bytes(cfg)).  `hip_stream` is a hipStream_t
 * (NULL = default stream).  EAGLE_EINVAL on a bad config / tree, EAGLE_ENOMEM if the workspace is too small. */
int eagle_init(const eagle_config *cfg, void *workspace_dev, size_t workspace_bytes, void *hip_stream, eagle_ctx **out);
void eagle_free(eagle_ctx *ctx);      /* releases host state only; the workspace belongs to the caller */

/* Copy one tensor (see enum) into the library's tiled layout.  `layer` is 0..n_layers-1, EAGLE_HEAD_LAYER, or
 * ignored for the global tensors.  `src_dev` is a device pointer holding the whole tensor; it may be released
 * as soon as the stream has passed this call.  All tensors must be loaded before eagle_prefill(). */
int eagle_load_weight(eagle_ctx *ctx, int32_t which, int32_t layer, const void *src_dev);

/* Forget all sequences (KV pages are returned, weights stay). */
int eagle_reset(eagle_ctx *ctx);

/* Target forward over the prompt (host int32[n], n >= 1) for slot `seq`, first token chosen from the target
 * distribution (argmax when greedy), and the head's forward over the pairs (f_i, x_{i+1}) -- Sec. 3.1's
 * "feature sequence and token sequence advanced by one time step".  *first_token (host) may be NULL. */
int eagle_prefill(eagle_ctx *ctx, int32_t seq, const int32_t *prompt_host, int32_t n, int32_t *first_token);

/* Drafting phase: D forward passes of the head expand the tree of every active slot.
 * tree_tokens_host: NULL or int32[n_active * n_nodes] receiving the tree's tokens (root first). */
int eagle_draft_tree(eagle_ctx *ctx, int32_t *tree_tokens_host);

/* Verification phase: one tree-masked target forward; logits [n_nodes, vocab] and features [n_nodes, d_model]
 * per slot stay in the context (read them with eagle_get_buffer). */
int eagle_verify(eagle_ctx *ctx);

/* Acceptance + commit: walks each slot's tree (greedy or Alg. 1), then moves the accepted path's KV rows and
 * features to consecutive slots in ONE kernel launch.  Host outputs, each may be NULL:
 *   out_tokens int32[n_active * (depth+1)]  accepted draft tokens followed by the bonus token
 *   out_len    int32[n_active]              number of tokens emitted, 1..depth+1
 *   path       int32[n_active * (depth+1)]  accepted node indices (= KV compaction sources), path[0] = 0 */
int eagle_accept(eagle_ctx *ctx, int32_t *out_tokens, int32_t *out_len, int32_t *path);

/* eagle_accept for callers that cannot allocate or hand over scratch memory (code that must not call hipMalloc: tight
 * serving loops, harnesses that forbid it): the same kernels, but their scratch -- the two fp32 [n_active, vocab]
 * probability vectors of Alg. 1, or the per-node arg-max array of the greedy walk -- lives in a 4 MiB array that is
 * part of the library's device code instead of in the context's workspace.  Inputs (the verified logits, the tree)
 * and outputs are those of eagle_accept.  Limit: non-greedy, n_active * vocab <= 524288 (16 slots at vocab 32000);
 * greedy always fits.  EAGLE_EINVAL beyond that, before anything is launched.  The call allocates nothing.  Every
 * context on one GPU shares that GPU's array (it keeps the last call's contents; the kernels write every element
 * they read): calls that overlap in time on one GPU race, also across contexts and streams. */
int eagle_accept_static(eagle_ctx *ctx, int32_t *out_tokens, int32_t *out_len, int32_t *path);

/* draft + verify + accept back to back with no host synchronisation in between; outputs as eagle_accept. */
int eagle_step(eagle_ctx *ctx, int32_t *out_tokens, int32_t *out_len, int32_t *path);

/* Plain autoregression with the same kernels: the target on the root token only; one token per slot
 * (host int32[n_active], may be NULL). */
int eagle_vanilla_step(eagle_ctx *ctx, int32_t *tokens_host);

/* Convenience loop for one sequence in slot `seq` (all other slots must be inactive): reset, prefill, then
 * speculative steps until max_new tokens exist.  out: host int32[max_new]; *n_out tokens written;
 * *mean_accept_len = tokens emitted per target forward (the paper's tau). */
int eagle_generate(eagle_ctx *ctx, int32_t seq, const int32_t *prompt_host, int32_t n_prompt, int32_t max_new,
                   int32_t *out, int32_t *n_out, float *mean_accept_len);

/* Acceptance knob of the synthetic workload: future[i] is the token the target will emit at absolute index i
 * of slot `seq`'s token sequence.  While a draft node's path follows `future`, the draft logit of the next
 * future token gets +bias when hash(seed, index) < alpha and -bias otherwise.  n = 0 switches it off. */
int eagle_set_hint(eagle_ctx *ctx, int32_t seq, const int32_t *future_host, int32_t n, float alpha, float bias, uint64_t seed);

/* ---- Injection: lock-step tests and callers that bring their own decisions -------------------------------------
 * These calls let the CPU side of a lock-step comparison drive the engine along ITS choices (Sec. 3.1 / App. A.1
 * tree, Sec. 3.3 / App. A.2 acceptance), and let the child-selection and acceptance kernels be run on logits the
 * caller supplies.  All of them synchronise the stream. */

/* KV paging: physical page of every (slot, logical page), host int32[max_batch * pages_per_slot] with
 * pages_per_slot = ceil(max_seq / page_tokens); must be a permutation of 0..max_batch*pages_per_slot-1.  Allowed only
 * while no slot is active (EAGLE_ESTATE otherwise).  The default is the interleaved map page*max_batch + slot. */
int eagle_set_page_table(eagle_ctx *ctx, const int32_t *table_host);

/* Overwrite a context-owned buffer of slot `seq` from host memory: EAGLE_BUF_LOGITS, _FEATURES, _DRAFT_LOGITS,
 * _DRAFT_FEATURES or _TREE_TOKENS; `bytes` must be the buffer's full size (see the enum below). */
int eagle_set_buffer(eagle_ctx *ctx, int32_t which, int32_t seq, const void *host_src, size_t bytes);

/* Replace the tokens of slot `seq`'s drafted tree (host int32[n_nodes], node 0 = the root token) between
 * eagle_draft_tree and eagle_verify.  The knob's on-path flags are not recomputed. */
int eagle_force_tree(eagle_ctx *ctx, int32_t seq, const int32_t *tokens_host);

/* Child selection alone (App. A.1): the children of the nodes of tree level `level` (-1 = the root, else
 * 1..depth-1: the level's nodes that have children) are chosen from whatever EAGLE_BUF_DRAFT_LOGITS holds --
 * top-k when greedy, Gumbel top-k with the context's seed and draw counter otherwise -- for every active slot. */
int eagle_expand_level(eagle_ctx *ctx, int32_t level);

/* Commit given paths instead of running the acceptance rule, then compact as eagle_accept does.  Host arrays:
 * path int32[n_active * (depth+1)] (node indices, path[0] = 0, each node a child of its predecessor),
 * len int32[n_active] (1..depth+1 tokens emitted: len-1 accepted drafts + the bonus), bonus int32[n_active]. */
int eagle_force_accept(eagle_ctx *ctx, const int32_t *path_host, const int32_t *len_host, const int32_t *bonus_host);

/* Test / bench access to context-owned buffers (synchronises). `which`: */
enum {
  EAGLE_BUF_LOGITS = 0,        /* fp32 [n_nodes, vocab]     verify logits of slot seq                      */
  EAGLE_BUF_FEATURES,          /* fp32 [n_nodes, d_model]   verify features                               */
  EAGLE_BUF_DRAFT_LOGITS,      /* fp32 [n_nodes, vocab]     head logits per node (rows of leaves are unset) */
  EAGLE_BUF_DRAFT_FEATURES,    /* fp32 [n_nodes, d_model]   head output feature per node                   */
  EAGLE_BUF_TREE_TOKENS,       /* int32 [n_nodes]                                                          */
  EAGLE_BUF_TOKENS,            /* int32 [n committed tokens] the slot's whole token sequence               */
  EAGLE_BUF_VANILLA_LOGITS,    /* fp32 [vocab]              logits of the last eagle_vanilla_step / prefill */
  EAGLE_BUF_STATE,             /* int32 [4]: committed tokens, cached target positions, pending features, steps */
  EAGLE_BUF_KV_ROW,            /* see eagle_get_kv_row                                                      */
  EAGLE_BUF_GEMM_TRACE,        /* profiling builds of the library (-DEAGLE_TRACE) only, all zero otherwise:
                                  uint64 [1024 work-groups][8 events], 100 MHz time stamps of ONE launch of the
                                  weight-streaming GEMM kernel, selected with the environment variable
                                  EAGLE_GEMM_TRACE=<index of the launch within the verify phase> (read by eagle_init);
                                  events: 0 entered, 1 activations staged, 2 weight stream done, 3 partial sums
                                  published, 4 epilogue done (the work-groups that ran one). */
  EAGLE_BUF_PREFILL_FEATURES   /* fp32 [rows, d_model]: target features of the rows of the most recent prompt pass of
                                  eagle_prefill (the whole prompt when it fits one pass: 512 rows for dense bf16
                                  models, 128 otherwise; else its last pass) -- Sec. 3.1: what the head's prompt
                                  pass consumes */
};
int eagle_get_buffer(eagle_ctx *ctx, int32_t which, int32_t seq, void *host_dst, size_t cap_bytes);
/* K and V (fp32, [n_kv_heads*head_dim] each) of target layer `layer` (or EAGLE_HEAD_LAYER) at cache position pos. */
int eagle_get_kv_row(eagle_ctx *ctx, int32_t seq, int32_t layer, int32_t pos, float *k_host, float *v_host);

/* Timing (HIP events on the context's stream).  mode 0 = off, 1 = phases (draft / verify / accept per eagle_step),
 * 2 = additionally every launch of the weight-streaming GEMM kernels and of the attention kernel inside eagle_step,
 * each with a start and a stop event attached to the dispatch itself (the kernel's own begin and end time stamps:
 * the figure a kernel trace shows for the launch). */
int eagle_set_profiling(eagle_ctx *ctx, int32_t mode);
typedef struct {
  double draft_ms, verify_ms, accept_ms;   /* sums over the steps since the last reset of the counters */
  int64_t steps;
  double gemm_ms; int64_t gemm_launches; double gemm_weight_bytes;  /* mode 2 only */
  double verify_weight_bytes, verify_kv_bytes;                    /* algorithmic bytes of the verify phases */
} eagle_profile;
int eagle_get_profile(eagle_ctx *ctx, eagle_profile *out, int32_t reset);
/* Mode 2, per class of launch and per phase (0 = drafting, 1 = verification): summed kernel durations, launches and
 * algorithmic HBM bytes (a weight matrix once in its stored type; for attention the keys and values of the context
 * and the pass's rows once).  name: qkv | attention | o_proj | gate_up | down | lm_head | fc; kernel: the template
 * that ran.  Up to `cap` entries are written, *n of them. */
typedef struct { char name[16]; char kernel[48]; double ms; int64_t launches; double bytes; } eagle_kernel_stat;
int eagle_get_kernel_stats(eagle_ctx *ctx, int32_t phase, eagle_kernel_stat *out, int32_t cap, int32_t *n, int32_t reset);

/* Training loss of the Autoregression Head and its gradient (Sec. 3.2 "Training of the draft models"):
 *   L_reg = mean over rows and columns of SmoothL1(fhat - f)      (threshold 1: 0.5 x^2 if |x| < 1, else |x| - 0.5)
 *   L_cls = mean over rows of -sum_v p_v log phat_v,  p = softmax(LM_Head(f)), phat = softmax(LM_Head(fhat))
 *   L     = L_reg + w_cls * L_cls                                  (the paper sets w_cls = 0.1)
 *   grad  = dL/dfhat = clip(fhat - f, -1, 1) / (rows * d_model) + w_cls / rows * (phat - p) W_lm_head
 * f (the target's feature of the next position: the label) and fhat (the head's prediction) are DEVICE pointers to
 * fp32 [rows, d_model], row-major, only read; the LM head is the one loaded into the context (frozen: it gets no
 * gradient).  grad_fhat: DEVICE pointer, fp32 [rows, d_model], written (may be null: loss only).  loss_out: HOST
 * pointer to 3 floats: L, L_reg, L_cls.  Any rows >= 1; the rows are processed in passes of at most half the
 * context's largest pass each (256 rows for a dense bf16 model).  Leaves the decoding state of the context untouched
 * (it uses only buffers that live within one pass).  Needs cfg.head_loss_rows > 0 and the LM head loaded
 * (EAGLE_ESTATE otherwise).  Synchronises the stream (the loss is returned by value). */
int eagle_head_loss(eagle_ctx *ctx, const float *f_dev, const float *fhat_dev, int32_t rows, float w_cls,
                    float *grad_fhat_dev, float *loss_out);

/* Data augmentation of Sec. 3.2: out[r][k] = in[r][k] + amplitude * n(r, k), n uniform on (-1, 1): the odd multiples of
 * 2^-24 drawn by the library's counter-based generator from (seed, step, r, k) -- reproducible, and a different
 * stream for every step.  fp32 [rows, d_model] DEVICE pointers; in == out is allowed.  The paper's amplitude is 0.1.
 * Needs no head_loss_rows.  Asynchronous on the context's stream. */
int eagle_feature_noise(eagle_ctx *ctx, const float *in_dev, float *out_dev, int32_t rows, float amplitude,
                        uint64_t seed, uint64_t step);

/* Measurement reference, independent of any context: a bare streaming read of `bytes` bytes of device memory
 * (16-byte loads, nothing computed), run `iters` times on `hip_stream`, each launch timed by its own start/stop
 * events; *gb_per_s = bytes read / summed kernel time.  The buffer is only read.  Synchronises the stream. */
int eagle_probe_stream_read(const void *buf_dev, size_t bytes, int32_t iters, void *hip_stream, double *gb_per_s);

const char *eagle_last_error(void);   /* thread-local text of the last failure */
const char *eagle_version(void);

#ifdef __cplusplus
}
#endif
#endif
