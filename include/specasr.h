/*
 * specasr.h -- C ABI of the MI355X (gfx950) tree-verification library.
 *
 * What it computes.  One verification round of SpecASR's speculative decoding:
 * the target LLM decoder evaluates every token of a sparse draft token tree in a
 * single pass against a KV cache that already holds the audio-embedding prefix,
 * the prompt and the accepted tokens (Sec. II-A: audio embeddings are prefilled
 * with the text prompt; Sec. II-B: tree verification with a 2D attention mask so
 * that each branch is verified independently; Sec. IV-C: the two-pass sparse
 * tree is verified with that mask), then accepts the draft tokens that match the
 * target's own greedy output and stops at the first failure (Sec. II-B,
 * "Draft-then-Verify"), and appends the accepted path to the cache.
 *
 * Conventions.
 *  - Every function returns a specasr_status; nothing throws or aborts.
 *  - "device" pointers are HIP device memory of the current device; "host"
 *    pointers are ordinary host memory.  The caller owns every buffer it passes
 *    (weights, KV cache, workspace, logits); they are borrowed for the call, the
 *    weights for the life of the context.  The library allocates device memory
 *    only inside specasr_create (the optional repacked weight copy).  Host-side
 *    resources are created by the first call that needs them and released by
 *    specasr_destroy: a few KB of pinned staging memory with one event per
 *    staging slot (any call that uploads tree metadata), up to three internal
 *    streams of default priority with fork/join events (calls that fall into
 *    several sequence groups, chunked prefill) plus two events per layer
 *    (chunked prefill), and event pairs for specasr_profile_stage.
 *  - The library reads no environment variable after specasr_create.  That
 *    call reads the development aids SPECASR_LANES, SPECASR_GEMM_SPLITS,
 *    SPECASR_WIDE_SPLITS, SPECASR_ATTN_CHUNK and SPECASR_DEBUG once (forced kernel
 *    plans for sweeps, diagnostics on stderr); results do not depend on them
 *    beyond summation order, and a deployment sets none.
 *  - `stream` is a raw hipStream_t (NULL = the default stream).
 *  - A context is not thread-safe, and calls that use the same workspace must not overlap on
 *    the device: issue them on one stream, or order them with events.  Calls on different
 *    contexts (e.g. a draft and a target model) with their own workspaces are independent.
 *  - All validation happens on the host before anything is enqueued: a call that
 *    returns an error has not touched the cache, kv_len or any output.
 *  - Tree convention.  Node 0 of a tree is the last committed token whose K/V is
 *    not yet in the cache (the previous round's next_token, or the last prompt
 *    token); it is always accepted.  parents[0] = -1 and 0 <= parents[i] < i.
 *    Node i is evaluated at position kv_len + depth(i) and its K/V is written to
 *    cache SLOT kv_len + i; it attends to slots [0, kv_len) and to the nodes on
 *    its own root path, itself included.
 *  - Matrices are row-major [out_features][in_features]; no biases.
 *  - Model: pre-norm Llama-style block (RMSNorm, rotary embedding with the
 *    rotate-half pairing and angle pos * theta^(-2j/head_dim), grouped-query
 *    attention with query head a using KV head a / (n_heads / n_kv_heads),
 *    SwiGLU feed-forward, untied LM head); the decoder family the paper targets
 *    (Sec. II-A, Sec. V-A).
 */
#ifndef SPECASR_H
#define SPECASR_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  SPECASR_OK = 0,
  SPECASR_E_NULL = -1,        /* a required pointer is NULL */
  SPECASR_E_CONFIG = -2,      /* inconsistent or unsupported model configuration */
  SPECASR_E_TREE = -3,        /* n_nodes out of range, bad parent array, token out of range */
  SPECASR_E_KV_OVERFLOW = -4, /* kv_len < 0 or kv_len + n_nodes > capacity */
  SPECASR_E_WORKSPACE = -5,   /* workspace missing, misaligned or too small */
  SPECASR_E_HIP = -6,         /* a HIP runtime call failed (see specasr_last_hip_error) */
  SPECASR_E_UNSUPPORTED = -7, /* valid request this build cannot serve */
  SPECASR_E_PATH = -8         /* commit: path is not a root path of the tree's size */
} specasr_status;

typedef enum { SPECASR_F32 = 0, SPECASR_BF16 = 1 } specasr_dtype;

/* flags for specasr_config.flags */
#define SPECASR_FLAG_GENERIC_KERNELS 1u /* force the dtype-generic kernels (no MFMA path) */
#define SPECASR_FLAG_NO_REPACK 2u       /* never make a repacked copy of the weights */
#define SPECASR_FLAG_NO_WIDE 4u         /* no buffers for passes over more than 64 rows: such calls run as
                                           groups of whole sequences, long prefills as chunks */

#define SPECASR_MAX_NODES 64 /* one wavefront lane / one mask bit per tree node */

typedef struct {
  int32_t n_layers, d_model, n_heads, n_kv_heads, head_dim, d_ffn, vocab;
  float rms_eps;      /* RMSNorm epsilon (added to the mean square)            */
  float rope_theta;   /* rotary base                                           */
  int32_t dtype;      /* specasr_dtype of weights AND KV cache                 */
  int32_t max_nodes;  /* largest tree per sequence, 1..SPECASR_MAX_NODES       */
  int32_t max_batch;  /* largest number of sequences per call, >= 1            */
  uint32_t flags;     /* SPECASR_FLAG_*                                        */
} specasr_config;

/* device pointers, storage type = config.dtype */
typedef struct {
  const void *attn_norm;                /* [d_model]                          */
  const void *wq;                       /* [n_heads*head_dim][d_model]        */
  const void *wk, *wv;                  /* [n_kv_heads*head_dim][d_model]     */
  const void *wo;                       /* [d_model][n_heads*head_dim]        */
  const void *ffn_norm;                 /* [d_model]                          */
  const void *w_gate, *w_up;            /* [d_ffn][d_model]                   */
  const void *w_down;                   /* [d_model][d_ffn]                   */
} specasr_layer_weights;

typedef struct {
  const void *tok_embed;                /* device [vocab][d_model]            */
  const void *final_norm;               /* device [d_model]                   */
  const void *lm_head;                  /* device [vocab][d_model]            */
  const specasr_layer_weights *layers;  /* HOST array [n_layers] of device pointers */
} specasr_weights;

/* KV cache: device, [batch][n_layers][n_kv_heads][capacity][head_dim], K rows are
 * stored after the rotary embedding.  Mutated by forward (slots kv_len..kv_len+n-1)
 * and by commit.  After verify, slots [kv_len_new, old kv_len + n) are scratch. */
typedef struct {
  void *k, *v;
  int64_t capacity;   /* slots per sequence                                   */
  int32_t batch;      /* sequences in the cache; tree.batch must equal it     */
  int32_t *kv_len;    /* HOST int32[batch]: read on entry, advanced by verify/commit on success */
} specasr_kv;

/* Draft token trees, one per sequence; HOST arrays with row stride max_nodes. */
typedef struct {
  const int32_t *tokens;   /* [batch][max_nodes]                              */
  const int32_t *parents;  /* [batch][max_nodes]                              */
  const int32_t *n_nodes;  /* [batch], each 1..max_nodes                      */
  /* Optional (prefill of audio-embedding positions, Sec. II-A): device array
   * [batch][max_nodes][d_model] in config.dtype and HOST flags [batch][max_nodes];
   * where a flag is non-zero the node's input row is taken from input_embeds
   * instead of the token embedding (its token is ignored).  Both NULL otherwise. */
  const void *input_embeds;
  const uint8_t *use_embed;
} specasr_tree;

/* Results of a verification round; HOST arrays except logits. */
typedef struct {
  int32_t *argmax;      /* [batch][max_nodes]: target's greedy token after each node */
  int32_t *path;        /* [batch][max_nodes]: accepted node indices, root first     */
  int32_t *accept_len;  /* [batch]: number of accepted nodes, >= 1 (root included)   */
  int32_t *next_token;  /* [batch]: argmax at the last accepted node                 */
  float *logits;        /* optional DEVICE fp32 [batch][max_nodes][vocab], or NULL   */
} specasr_out;

typedef struct specasr_ctx specasr_ctx;

/* Create a context for one model on the current HIP device.  Validates the
 * configuration (E_CONFIG), may copy weights into a streaming-friendly layout
 * unless SPECASR_FLAG_NO_REPACK (values unchanged bit for bit).  The weight
 * pointers must stay valid until specasr_destroy. */
specasr_status specasr_create(const specasr_config *cfg, const specasr_weights *weights,
                              specasr_ctx **out);
void specasr_destroy(specasr_ctx *ctx);

/* Bytes of device workspace a call with `batch` sequences needs (256-byte aligned
 * base required).  Depends on the model, max_nodes and batch only.  On the bf16 MFMA path it
 * covers one set of buffers per internal stream plus one set for passes over up to
 * max(16, batch) x max_nodes rows (prefill, large batches). */
size_t specasr_workspace_bytes(const specasr_ctx *ctx, int32_t batch);

/* One whole verification round (Sec. II-B, Sec. IV-C): tree forward, per-node
 * greedy argmax, acceptance of the longest matching path, in-place compaction of
 * the accepted nodes' K/V to slots kv_len..kv_len+accept_len-1.  Synchronises the
 * stream once before returning so that the host outputs are valid; on success
 * kv->kv_len[b] += accept_len[b]. */
specasr_status specasr_verify_tree(specasr_ctx *ctx, specasr_kv *kv, const specasr_tree *tree,
                                   specasr_out *out, void *workspace, size_t workspace_bytes,
                                   void *stream);

/* Stage: decoder forward over the tree tokens only (the single-pass tree
 * verification of Sec. II-B).  Writes K/V of node i to slot kv_len+i, the greedy
 * token per node to argmax_dev (DEVICE int32 [batch][max_nodes]) and, if
 * logits_dev != NULL, fp32 logits [batch][max_nodes][vocab].  Asynchronous;
 * kv_len is not changed. */
specasr_status specasr_tree_forward(specasr_ctx *ctx, specasr_kv *kv, const specasr_tree *tree,
                                    int32_t *argmax_dev, float *logits_dev, void *workspace,
                                    size_t workspace_bytes, void *stream);

/* Draft-side tree forward (Sec. IV-B: the draft model runs on a masked token tree -- the old draft
 * as one branch, the part being regenerated as the other -- so that regeneration and reuse
 * proceed in one pass; Sec. IV-A: the normalised logit of each predicted token is compared with
 * a threshold; Sec. IV-C: positions of low confidence keep the tokens of highest probability and
 * the second one is expanded).  Same kernels and the same semantics as specasr_tree_forward (the
 * K/V rows of the nodes are written to slots kv_len + node, kv_len itself is unchanged), with a
 * different read-out per node:
 *   top2_dev      DEVICE int32 [batch][max_nodes][2]: ids of the largest and the second largest
 *                 logit (value descending, lower id first among equal values; the second is -1
 *                 for a one-token vocabulary); entries of nodes >= n_nodes are not written
 *   top1_prob_dev DEVICE float [batch][max_nodes]: softmax probability of the first id
 *   logits_dev    optional DEVICE fp32 [batch][max_nodes][vocab], or NULL
 * Asynchronous on `stream`; errors as specasr_tree_forward. */
specasr_status specasr_tree_forward_top2(specasr_ctx *ctx, specasr_kv *kv, const specasr_tree *tree,
                                         int32_t *top2_dev, float *top1_prob_dev, float *logits_dev,
                                         void *workspace, size_t workspace_bytes, void *stream);

/* Prefill (Sec. II-A: the audio embeddings produced by the speech encoder are prefilled alongside
 * the text prompt; the verify rounds then run against that cache).  Appends n_pos[b] positions to
 * every sequence b: position i takes the embedding row input_embeds[b][i] where use_embed[b][i] is
 * non-zero, the token embedding of tokens[b][i] otherwise.  The positions are run through the
 * decoder in chain-shaped chunks of at most max_nodes rows (a chain is the tree whose mask is the
 * causal one) -- on the bf16 MFMA path a sequence that adds more than max_nodes positions takes
 * up to 16 consecutive chunks at once, as one pass over up to 16 x max_nodes rows whose projections
 * are matrix-core-bound GEMMs -- their K/V rows land in slots kv_len .. kv_len + n_pos - 1, and
 * kv_len advances by n_pos.  The LM head runs only for the last chunk, and only if next_token is
 * given.
 *   tokens        HOST int32 [batch][max_pos], may be NULL if every position is an embedding
 *   input_embeds  DEVICE [batch][max_pos][d_model] in config.dtype, with use_embed HOST uint8
 *                 [batch][max_pos]; both NULL when every position is a token
 *   n_pos         HOST int32 [batch], each 0..max_pos
 *   next_token    optional HOST int32 [batch]: the model's greedy token after the last position
 *                 (-1 for a sequence with n_pos = 0); when given the call synchronises the stream
 * Errors: E_NULL, E_TREE (token id or n_pos out of range), E_KV_OVERFLOW, E_WORKSPACE; nothing is
 * enqueued and kv_len is unchanged on error. */
specasr_status specasr_prefill(specasr_ctx *ctx, specasr_kv *kv, const int32_t *tokens,
                               const void *input_embeds, const uint8_t *use_embed,
                               const int32_t *n_pos, int32_t max_pos, int32_t *next_token,
                               void *workspace, size_t workspace_bytes, void *stream);

/* Stage: greedy acceptance (Sec. II-B: accept matching draft tokens, stop at the
 * first failure) from a DEVICE argmax array.  A draft node matches when its token
 * equals the argmax at its parent; the result is the deepest node whose whole
 * root path matches (lowest index among equals).  Outputs are DEVICE arrays
 * path_dev [batch][max_nodes] (entries past accept_len are -1), accept_len_dev
 * [batch], next_token_dev [batch].  Asynchronous. */
specasr_status specasr_accept(specasr_ctx *ctx, const specasr_tree *tree, int32_t batch,
                              const int32_t *argmax_dev, int32_t *path_dev,
                              int32_t *accept_len_dev, int32_t *next_token_dev, void *workspace,
                              size_t workspace_bytes, void *stream);

/* Stage: per-node argmax (lowest token id on exact ties) of caller-supplied DEVICE
 * fp32 logits [batch][max_nodes][vocab], written to argmax_dev, followed by
 * specasr_accept on it.  Asynchronous. */
specasr_status specasr_accept_from_logits(specasr_ctx *ctx, const specasr_tree *tree,
                                          int32_t batch, const float *logits_dev,
                                          int32_t *argmax_dev, int32_t *path_dev,
                                          int32_t *accept_len_dev, int32_t *next_token_dev,
                                          void *workspace, size_t workspace_bytes, void *stream);

/* specasr_accept_from_logits for callers that cannot allocate: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same inputs, outputs, semantics and
 * validation, but no workspace argument: the flattened tree metadata the kernels read lives in a
 * device array of the library (40 KB, held by every GPU the library has run this call on until the
 * process ends), filled by a kernel that receives each tree in its arguments.  The call allocates
 * no device, pinned or host memory, copies nothing and does not synchronise; asynchronous on
 * `stream`.  Limit: batch <= SPECASR_STATIC_MAX_BATCH (E_UNSUPPORTED beyond it, nothing enqueued).
 * All calls on one GPU share the one array: calls that overlap on a GPU (other streams, other
 * contexts, other threads) race; order them on one stream or with events. */
#define SPECASR_STATIC_MAX_BATCH 16
specasr_status specasr_accept_from_logits_static(specasr_ctx *ctx, const specasr_tree *tree,
                                                 int32_t batch, const float *logits_dev,
                                                 int32_t *argmax_dev, int32_t *path_dev,
                                                 int32_t *accept_len_dev, int32_t *next_token_dev,
                                                 void *stream);

/* Stage: commit a path (the cache update that lets the next round start where
 * the accepted tokens end): for k < accept_len[b], cache slot kv_len+path[k] is
 * moved to slot kv_len+k for every layer and KV head, K and V, in place; then
 * kv->kv_len[b] += accept_len[b].  path/accept_len are HOST arrays with row stride
 * max_nodes; path[b][0] must be 0 and the path strictly increasing.  n_nodes
 * (HOST [batch]) bounds the indices.  Asynchronous on the device. */
specasr_status specasr_commit(specasr_ctx *ctx, specasr_kv *kv, const int32_t *n_nodes,
                              const int32_t *path, const int32_t *accept_len, void *workspace,
                              size_t workspace_bytes, void *stream);

/* Which kernels a forward over `rows` tree nodes in total would use: 1 = the bf16 MFMA path
 * (a call with more than 64 rows runs as a single pass with its projections on the tiled
 * large-M GEMM; where the head size has no MFMA attention, as consecutive groups of whole
 * sequences with at most 64 rows each), 0 = the dtype-generic kernels (fp32 models, SPECASR_FLAG_GENERIC_KERNELS /
 * NO_REPACK, shapes the MFMA tiling does not cover). */
int32_t specasr_uses_mfma(const specasr_ctx *ctx, int32_t rows);

const char *specasr_strerror(specasr_status s);
/* hipError_t value of the last failing HIP call seen by this context (0 if none). */
int32_t specasr_last_hip_error(const specasr_ctx *ctx);
/* Library/ABI version, bumped when a signature or struct changes. */
int32_t specasr_abi_version(void);

#ifdef __cplusplus
}
#endif
#endif /* SPECASR_H */
