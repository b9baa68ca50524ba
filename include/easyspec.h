/*
 * easyspec.h — C ABI of the MI355X (gfx950) EasySpec draft-model hot path.
 *
 * What the library computes (EasySpec, arXiv 2502.02493):
 *   - easyspec_draft_step     one layer-parallel "fuzzy" forward of the draft model
 *                             (paper Alg. 2; the layer-parallel strategy of Sec. 3.1.1)
 *   - easyspec_draft_tree_step  the same fuzzy forward over one level of a token tree (App. C)
 *   - easyspec_calibrate      bonus calibration: drop the fuzzy KV entries, refill the cache
 *                             with precise values by one token-parallel, layer-sequential
 *                             forward (paper Sec. 3.2, Alg. 1)
 *   - easyspec_greedy_accept  acceptance of drafted tokens at temperature 0 (paper Alg. 3)
 *   - easyspec_accept         acceptance by speculative sampling at a temperature > 0
 *                             (paper Alg. 3, bonus distribution of Sec. 2.1)
 *
 * Model function: pre-norm decoder with RMSNorm, rotary embedding (pairs i, i + head_dim/2),
 * grouped-query attention (query head j reads KV head j / (n_q_heads/n_kv_heads)), SwiGLU MLP,
 * untied LM head.  Storage dtype (weights and KV cache) is fp32 or bf16; the residual stream,
 * queries, softmax and all accumulators are fp32.
 *
 * Conventions
 *   - Every function returns EASYSPEC_OK (0) or a negative error code.  Arguments are checked
 *     on the host before anything is launched: a failed call leaves lengths and device memory
 *     unchanged.  easyspec_last_error() returns a message for the last failure.
 *   - "dev" pointers are device memory owned by the caller; they must stay valid until the
 *     context's stream has passed the call.  "host" pointers are ordinary host memory.
 *     "host|dev" pointers may be either.  The library never frees caller memory.
 *   - Calls are asynchronous on the stream given at creation unless stated otherwise.
 *   - A context is not thread-safe; use one thread per context.
 *   - The library has no CPU fallback: without a usable HIP device easyspec_create fails.
 *   - Measurement and test hooks (per-kernel timing, the bandwidth probe, host models of the
 *     kernels' index arithmetic, workspace poisoning) are declared apart, in easyspec_instrument.h:
 *     no caller of the method needs them.
 */
#ifndef EASYSPEC_H
#define EASYSPEC_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define EASYSPEC_OK 0
#define EASYSPEC_EINVAL (-1)    /* bad argument or unsupported shape */
#define EASYSPEC_ECAPACITY (-2) /* a sequence would exceed max_ctx, or too many tokens */
#define EASYSPEC_ESTATE (-3)    /* call not valid in the current state (no weights, no live sequence, ...) */
#define EASYSPEC_EHIP (-4)      /* a HIP runtime call failed; message in easyspec_last_error */

#define EASYSPEC_DTYPE_F32 0
#define EASYSPEC_DTYPE_BF16 1

#define EASYSPEC_POLICY_ALIGNED 0 /* the rule in the text of Sec. 3.1.1 */
#define EASYSPEC_POLICY_PACKED 1  /* the 16-layer row of the strategy table of Sec. 3.1.1 */

#define EASYSPEC_MAX_BATCH 16        /* sequences per context */
#define EASYSPEC_MAX_CALIB_TOKENS 16 /* tokens of one sequence per calibration call */
#define EASYSPEC_MAX_SET 8           /* layers per layer-parallel set */
#define EASYSPEC_MAX_TREE_WIDTH 16   /* nodes one easyspec_draft_tree_step call may add (all sequences together) */
#define EASYSPEC_MAX_TREE_NODES 64   /* nodes of one sequence's token tree */

typedef struct easyspec_config {
  int32_t n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab;
  float rms_eps, rope_theta;
  int32_t qkv_bias;         /* 0/1: q, k, v projections carry a bias */
  int32_t dtype;            /* EASYSPEC_DTYPE_*: storage type of matrices, embedding and KV cache */
  int32_t max_batch;        /* 1..EASYSPEC_MAX_BATCH sequences */
  int32_t max_ctx;          /* KV slots per sequence (precise + fuzzy) */
  int32_t max_calib_tokens; /* 1..EASYSPEC_MAX_CALIB_TOKENS */
} easyspec_config;
/* Shape limits: head_dim is 64 or 128; d_model, n_q_heads*head_dim and d_ffn are multiples
 * of 32; n_q_heads/n_kv_heads is 1, 2, 4, 7 or 8. */

typedef struct easyspec_layer_weights {
  /* row-major [out][in] matrices in the storage dtype (bf16 = raw 16-bit patterns) */
  const void *wq; /* [n_q_heads*head_dim][d_model]  */
  const void *wk; /* [n_kv_heads*head_dim][d_model] */
  const void *wv; /* [n_kv_heads*head_dim][d_model] */
  const void *wo; /* [d_model][n_q_heads*head_dim]  */
  const void *wg; /* [d_ffn][d_model]  gate */
  const void *wu; /* [d_ffn][d_model]  up   */
  const void *wd; /* [d_model][d_ffn]  down */
  /* fp32 vectors */
  const float *bq, *bk, *bv; /* biases, NULL unless qkv_bias */
  const float *g_attn;       /* [d_model] gain of the norm before attention */
  const float *g_mlp;        /* [d_model] gain of the norm before the MLP */
} easyspec_layer_weights;

typedef struct easyspec_weights {
  const easyspec_layer_weights *layers; /* host array of n_layers entries */
  const void *embed;                    /* [vocab][d_model] storage dtype */
  const void *lm_head;                  /* [vocab][d_model] storage dtype */
  const float *g_final;                 /* [d_model] fp32 */
} easyspec_weights;

typedef struct easyspec_ctx easyspec_ctx; /* opaque: owns its weight copy, KV cache and workspaces */

/* Create a context on the current HIP device.  hip_stream: a hipStream_t (NULL = the default
 * stream) on which every later call is ordered.  Allocates the packed weight arrays, the KV
 * cache ([layer][sequence][kv_head][slot][head_dim], K and V apart) and the workspaces; the
 * rotary table is computed on the host in double precision.  Starts with every layer in a set
 * of its own (plain sequential order, paper Alg. 1).  *out is NULL on failure. */
int easyspec_create(const easyspec_config *cfg, void *hip_stream, easyspec_ctx **out);

/* Frees everything the context owns (synchronises its stream first).  NULL is allowed. */
void easyspec_destroy(easyspec_ctx *ctx);

/* Copy the parameters into the context, repacked into the library's streaming layout: per
 * operation one layer-major array, so that the layers of any set are one contiguous range.
 * Every pointer inside src is host|dev; the caller keeps src.  Synchronous. */
int easyspec_load_weights(easyspec_ctx *ctx, const easyspec_weights *src);

/* Layer-parallel strategy (Sec. 3.1.1: the strategy is a configuration choice, no retraining).
 * bounds (host): bounds[0] = 0 < bounds[1] < ... < bounds[n_sets] = n_layers; set j is the
 * layers [bounds[j], bounds[j+1]), at most EASYSPEC_MAX_SET of them.  Only fuzzy steps use it. */
int easyspec_set_groups(easyspec_ctx *ctx, const int32_t *bounds, int32_t n_sets);

/* Boundaries of the paper's strategy for layer-parallel size N: first and last layer alone,
 * the layers between cut into N-sets (policy: see EASYSPEC_POLICY_*).  bounds (host) must hold
 * n_layers + 1 entries; *n_sets receives the number of sets.  Pure host function. */
int easyspec_default_groups(int32_t n_layers, int32_t N, int32_t policy, int32_t *bounds, int32_t *n_sets);

/* What the layers of a set share in fuzzy steps (easyspec_draft_step, easyspec_draft_tree_step).
 *   EASYSPEC_PARALLEL_ATTENTION (default)  Alg. 2: the attention layers of a set read the set's
 *       input; the MLPs run in layer order on the running residual.
 *   EASYSPEC_PARALLEL_FULL_LAYER  the ablation of App. B: attention AND MLP of every layer of the
 *       set work from the set's input h_1: a_i = Attn_i(h_1), m_i = MLP_i(h_1 + a_i),
 *       output = h_1 + sum_i (a_i + m_i).  The paper reports this variant as worse and does not
 *       define it; this is the reading "each layer of the set runs whole from the same input".
 * Sets of one layer are Alg. 1 in both modes.  Calibration is unaffected.  EASYSPEC_EINVAL for
 * an unknown mode. */
#define EASYSPEC_PARALLEL_ATTENTION 0
#define EASYSPEC_PARALLEL_FULL_LAYER 1
int easyspec_set_parallel_mode(easyspec_ctx *ctx, int32_t mode);

/* One fuzzy forward (Alg. 2) for every live sequence (precise length > 0), one token each.
 *   tokens_in  dev [max_batch]  token fed to sequence b (ignored for idle sequences)
 *   tokens_out dev [max_batch]  argmax of the logits, lowest index on ties (idle: untouched)
 *   logits_out dev [max_batch][vocab] fp32, or NULL
 * For each set, every attention layer of the set reads the hidden state entering the set and
 * stores the k, v it computes from it in slot precise+fuzzy; the MLPs run in layer order.
 * Afterwards fuzzy[b] += 1.  EASYSPEC_ESTATE if no sequence is live, EASYSPEC_ECAPACITY if a
 * live sequence is full. */
int easyspec_draft_step(easyspec_ctx *ctx, const int32_t *tokens_in, int32_t *tokens_out, float *logits_out);

/* One fuzzy forward (Alg. 2) over one level of a token tree (Sec. 3.1 last paragraph, App. C):
 * the drafted tokens of a sequence form a tree, every root-to-node path being one candidate
 * sequence; common prefixes share their KV entries and a node attends to the precise context,
 * its ancestors and itself (its row of the 2-D tree mask).  How the tree is grown (which tokens
 * become children of which node) is the caller's policy; the paper fixes none.
 *   tokens_in   dev  [max_batch][EASYSPEC_MAX_TREE_WIDTH]  tokens of the new nodes of sequence b
 *   n_nodes     host [max_batch]  number of new nodes of b, 0 = none; at most
 *                    EASYSPEC_MAX_TREE_WIDTH over all sequences
 *   parents     host [max_batch][EASYSPEC_MAX_TREE_WIDTH]  parent of new node j: a node index of b's
 *                    tree as it stood before the call (nodes are numbered in the order they were
 *                    added, 0 .. fuzzy[b]-1), or -1 = child of the last precise token
 *   tokens_out  dev  [max_batch][EASYSPEC_MAX_TREE_WIDTH]  argmax after each new node
 *   logits_out  dev  fp32 [max_batch][EASYSPEC_MAX_TREE_WIDTH][vocab] or NULL (for top-k children)
 * New node j of b takes slot precise[b] + fuzzy[b] + j in every layer (its k, v are those of the
 * fuzzy forward) and rotary position precise[b] + depth, depth = 0 for children of the last precise
 * token.  Afterwards fuzzy[b] += n_nodes[b].  A tree whose every node is the child of the previous
 * one is chain drafting.  Trees and easyspec_draft_step do not mix between two calibrations:
 * EASYSPEC_ESTATE if b holds chain-drafted slots (and easyspec_draft_step refuses a sequence that
 * holds a tree).  EASYSPEC_ECAPACITY beyond EASYSPEC_MAX_TREE_NODES nodes, max_ctx slots or the
 * per-call width; EASYSPEC_EINVAL for a parent that is not an earlier node.  Calibration drops
 * the whole tree like any fuzzy slots. */
int easyspec_draft_tree_step(easyspec_ctx *ctx, const int32_t *tokens_in, const int32_t *n_nodes, const int32_t *parents,
                             int32_t *tokens_out, float *logits_out);

/* Bonus calibration (Sec. 3.2) of the sequences with n_tokens[b] > 0; also the prompt prefill
 * (repeat in chunks of max_calib_tokens).
 *   tokens         dev  [max_batch][max_calib_tokens]  accepted tokens followed by the bonus token
 *   n_tokens       host [max_batch]  0 = leave sequence b alone, else 1..max_calib_tokens
 *   next_token_out dev  [max_batch]  argmax after the last token of b (untouched if n_tokens[b]=0)
 *   logits_out     dev  fp32 or NULL: logits_rows = 0 -> [max_batch][vocab] (last token of each);
 *                  logits_rows = 1 -> [max_batch][max_calib_tokens][vocab] (every token)
 * For each such sequence: fuzzy[b] = 0 (all fuzzy slots dropped, accepted or not); layers run
 * in order over the n tokens at positions precise[b] .. precise[b]+n-1, causal among themselves;
 * their k, v overwrite those slots; precise[b] += n.
 * A forward pass holds up to 16 token columns.  The sequences are taken in index order and packed into
 * passes, a sequence's tokens staying together; two consecutive passes of equal column counts run
 * together, each weight matrix being read once for both (so 4 sequences x 6 tokens cost one read of the
 * weights, not two); other passes run one after the other.  The results do not depend on the packing
 * beyond the last bits of fp32 arithmetic. */
int easyspec_calibrate(easyspec_ctx *ctx, const int32_t *tokens, const int32_t *n_tokens,
                       int32_t *next_token_out, float *logits_out, int32_t logits_rows);

/* Greedy acceptance (Alg. 3 with one-hot distributions): accept_len[b] = number of leading
 * positions where draft equals target_argmax; bonus[b] = target_argmax[b][accept_len[b]].
 *   draft [batch][gamma], target_argmax [batch][gamma+1], accept_len [batch], bonus [batch]
 * easyspec_greedy_accept: all four are dev arrays; one small kernel is launched on hip_stream (a
 * hipStream_t, NULL = the null stream, as everywhere in this header) and nothing is synchronised,
 * so the call is ordered with the draft steps that wrote `draft` on the same stream.
 * EASYSPEC_EINVAL for NULL pointers, batch < 1, gamma < 0, or an accept_len that is not device
 * memory (host arrays belong to the _host variant); EASYSPEC_EHIP without a HIP device.
 * easyspec_greedy_accept_host: all four are host arrays; a plain host loop, no device needed. */
int easyspec_greedy_accept(const int32_t *draft, const int32_t *target_argmax, int32_t batch, int32_t gamma,
                           int32_t *accept_len, int32_t *bonus, void *hip_stream);
int easyspec_greedy_accept_host(const int32_t *draft, const int32_t *target_argmax, int32_t batch, int32_t gamma,
                                int32_t *accept_len, int32_t *bonus);

/* Acceptance by speculative sampling (Alg. 3; Sec. 2.1) of `batch` sequences, in double
 * precision on the device, with the random numbers supplied by the caller.
 *   draft          dev [batch][gamma]            drafted tokens x'_i
 *   draft_logits   dev [batch][gamma][vocab]     fp32; p'_i = softmax(draft_logits[i] / temperature)
 *   target_logits  dev [batch][gamma+1][vocab]   fp32; p_i  = softmax(target_logits[i] / temperature)
 *   r              dev [batch][gamma]            uniforms in [0,1): position i is rejected when
 *                                                r_i > p_i(x'_i) / p'_i(x'_i)
 *   u              dev [batch]                   uniform in [0,1) for the bonus draw
 *   accept_len     dev [batch]  m = index of the first rejected position, or gamma
 *   bonus          dev [batch]  drawn from max(0, p_m - p'_m) normalised if m < gamma (the distributions
 *                               at the first rejected position), from p_gamma otherwise: the lowest token v
 *                               whose running sum over tokens 0..v exceeds u times the total
 *   workspace      dev, easyspec_accept_workspace_bytes(batch, gamma, vocab) bytes, 8-byte aligned
 *                  (about 8 bytes per vocabulary entry and sequence: the bonus weights);
 *                  contents need not be kept between calls
 *   hip_stream     the hipStream_t to launch on (NULL = the null stream); nothing is synchronised
 * gamma may be 0 (plain sampling from p_0).  A drafted token outside 0..vocab-1 at or before
 * the first rejected position gives accept_len = bonus = -1 for that sequence.  EASYSPEC_EINVAL for NULL pointers, batch < 1 or
 * > 65535, gamma outside 0..64, vocab < 1, or a temperature that is not positive and finite
 * (temperature 0 is easyspec_greedy_accept).  All arrays are the caller's and only read,
 * except accept_len, bonus and workspace. */
int easyspec_accept(const int32_t *draft, const float *draft_logits, const float *target_logits, const float *r,
                    const float *u, int32_t batch, int32_t gamma, int32_t vocab, float temperature,
                    int32_t *accept_len, int32_t *bonus, void *workspace, void *hip_stream);
int64_t easyspec_accept_workspace_bytes(int32_t batch, int32_t gamma, int32_t vocab); /* -1 for bad arguments */

/* easyspec_accept for callers that cannot allocate device memory and have no workspace to hand in
 * (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): same
 * arguments, same kernels and same results, but the workspace is the library's own fixed device
 * array of easyspec_accept_static_max_bytes() bytes (8 MiB; every GPU the library runs on holds one
 * until the process ends).  The call allocates and frees nothing.  EASYSPEC_ECAPACITY, with nothing
 * launched, when easyspec_accept_workspace_bytes(batch, gamma, vocab) exceeds that size (about 8
 * bytes per vocabulary entry and sequence: 6 sequences at a vocabulary of 152 064); other errors as
 * easyspec_accept.  All calls on one GPU share the array, so two calls whose kernels can overlap
 * (different streams, different threads) race: keep them on one stream, or order them yourself. */
int easyspec_accept_static(const int32_t *draft, const float *draft_logits, const float *target_logits, const float *r,
                           const float *u, int32_t batch, int32_t gamma, int32_t vocab, float temperature,
                           int32_t *accept_len, int32_t *bonus, void *hip_stream);
int64_t easyspec_accept_static_max_bytes(void);

/* Host copies of the per-sequence lengths; each of precise, fuzzy: host [max_batch] or NULL. */
int easyspec_get_lens(const easyspec_ctx *ctx, int32_t *precise, int32_t *fuzzy);

/* Shorten sequence b to new_precise_len precise slots and no fuzzy ones (base-model rollback
 * after verification; 0 makes the sequence idle).  Host state only. */
int easyspec_truncate(easyspec_ctx *ctx, int32_t b, int32_t new_precise_len);

/* Replace the cache of sequence b by n_slots precise entries.  k, v: host|dev
 * [n_layers][n_kv_heads][n_slots][head_dim] in the storage dtype.  Synchronous. */
int easyspec_kv_import(easyspec_ctx *ctx, int32_t b, const void *k, const void *v, int32_t n_slots);

/* Copy slots [0, n_slots) of sequence b out (same layout as import; fuzzy slots included if
 * n_slots reaches them).  Synchronous. */
int easyspec_kv_export(easyspec_ctx *ctx, int32_t b, void *k, void *v, int32_t n_slots);

/* Final residual-stream rows (before the last norm) of the most recent forward, in the order
 * the forward processed them (draft step: live sequences by index; calibration: sequences by
 * index, tokens in order).  out: dev fp32 [n_rows][d_model]; *n_rows (host) receives the count.
 * For parity checks of hidden states. */
int easyspec_get_hidden(easyspec_ctx *ctx, float *out, int32_t max_rows, int32_t *n_rows);

/* Algorithmic HBM bytes of one draft step in the current state: layer weights + LM head + the
 * KV slots each live sequence reads.  Pure host arithmetic, for roofline reports. */
int64_t easyspec_step_bytes(const easyspec_ctx *ctx);

/* Message of the last failed call on ctx (ctx == NULL: of the last failed easyspec_create or
 * context-free call on this thread).  Never NULL. */
const char *easyspec_last_error(const easyspec_ctx *ctx);

#ifdef __cplusplus
}
#endif
#endif /* EASYSPEC_H */
