// C ABI and host dispatcher of the tree-verification library (see include/specasr.h).
// Validates on the host, stages the tree metadata through pinned memory, enqueues the
// stages on the caller's stream.
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>
#include <vector>

#include "../../include/specasr.h"
#include "kernels.h"

using namespace specasr;

namespace {

constexpr int kStagingSlots = 8;

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

struct Staging {
  int32_t *host = nullptr;  // pinned
  hipEvent_t done = nullptr;
  bool used = false;
};

// offsets (in bytes) of the regions of a workspace sized for `rows_max` rows / `batch` sequences
struct WsLayout {
  size_t meta, outs, rope, x, h, q, k, v, att, gu, t, logits, total;
  size_t meta_words;
};

}  // namespace

struct specasr_ctx {
  specasr_config cfg;
  ModelDims md;
  specasr_weights w;
  std::vector<specasr_layer_weights> layers;
  Staging stage[kStagingSlots];
  int next_stage = 0;
  int32_t *out_host = nullptr;  // pinned, results of verify_tree
  size_t out_host_words = 0;
  int32_t last_hip = 0;
  int device = 0;
  bool staging_ready = false;
};

namespace {

#define HIP_TRY(ctx, expr)                                  \
  do {                                                      \
    hipError_t e_ = (expr);                                 \
    if (e_ != hipSuccess) {                                 \
      (ctx)->last_hip = (int32_t)e_;                        \
      return SPECASR_E_HIP;                                 \
    }                                                       \
  } while (0)

size_t meta_words(int rows_max, int batch) {
  // token, seq, node, depth, pos, slot, parent, use_embed: 8 words per row; anc: 2 words per row;
  // kv_len, row_start, n_nodes: 3 words per sequence
  return (size_t)rows_max * 10 + (size_t)batch * 3;
}

WsLayout ws_layout(const specasr_config &c, int batch) {
  WsLayout L{};
  const size_t R = (size_t)batch * c.max_nodes;
  const size_t dq = (size_t)c.n_heads * c.head_dim, dkv = (size_t)c.n_kv_heads * c.head_dim;
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, 256); return o; };
  L.meta_words = meta_words((int)R, batch);
  L.meta = take(L.meta_words * 4);
  L.outs = take(((size_t)batch * c.max_nodes * 2 + (size_t)batch * 2) * 4);  // argmax, path, len, next
  L.rope = take(R * (c.head_dim / 2) * sizeof(float2));
  L.x = take(R * c.d_model * 4);
  L.h = take(R * (c.d_model > (int)dq ? c.d_model : dq) * 4);
  L.q = take(R * dq * 4);
  L.k = take(R * dkv * 4);
  L.v = take(R * dkv * 4);
  L.att = take(R * dq * 4);
  L.gu = take(R * 2 * c.d_ffn * 4);
  L.t = take(R * c.d_ffn * 4);
  L.logits = take(R * c.vocab * 4);
  L.total = off;
  return L;
}

// Host-side view of one call: validated and flattened tree metadata.
struct HostStep {
  int rows = 0, batch = 0;
  std::vector<int32_t> words;  // the block copied to the device
};

specasr_status validate_tree(const specasr_ctx *ctx, const specasr_tree *tree, int batch,
                             const int32_t *kv_len, int64_t capacity, bool check_tokens) {
  const specasr_config &c = ctx->cfg;
  if (!tree || !tree->tokens || !tree->parents || !tree->n_nodes) return SPECASR_E_NULL;
  if ((tree->input_embeds == nullptr) != (tree->use_embed == nullptr)) return SPECASR_E_NULL;
  if (batch < 1 || batch > c.max_batch) return SPECASR_E_TREE;
  for (int b = 0; b < batch; ++b) {
    const int n = tree->n_nodes[b];
    if (n < 1 || n > c.max_nodes) return SPECASR_E_TREE;
    const int32_t *par = tree->parents + (size_t)b * c.max_nodes;
    const int32_t *tok = tree->tokens + (size_t)b * c.max_nodes;
    if (par[0] != -1) return SPECASR_E_TREE;
    for (int i = 1; i < n; ++i)
      if (par[i] < 0 || par[i] >= i) return SPECASR_E_TREE;
    if (check_tokens)
      for (int i = 0; i < n; ++i) {
        const bool emb = tree->use_embed && tree->use_embed[(size_t)b * c.max_nodes + i];
        if (!emb && (tok[i] < 0 || tok[i] >= c.vocab)) return SPECASR_E_TREE;
      }
    if (kv_len) {
      if (kv_len[b] < 0 || (int64_t)kv_len[b] + n > capacity) return SPECASR_E_KV_OVERFLOW;
    }
  }
  return SPECASR_OK;
}

// Step 0 of the path: depth and ancestor bit masks from the parent array, plus the flattened
// row tables.  kv_len may be NULL (acceptance only), then positions and slots are zero-based.
void build_step(const specasr_ctx *ctx, const specasr_tree *tree, int batch, const int32_t *kv_len,
                HostStep *hs) {
  const specasr_config &c = ctx->cfg;
  int rows = 0;
  for (int b = 0; b < batch; ++b) rows += tree->n_nodes[b];
  const int R = batch * c.max_nodes;
  hs->rows = rows;
  hs->batch = batch;
  hs->words.assign(meta_words(R, batch), 0);
  int32_t *w = hs->words.data();
  int32_t *token = w, *seq = w + R, *node = w + 2 * R, *depth = w + 3 * R, *pos = w + 4 * R,
          *slot = w + 5 * R, *parent = w + 6 * R, *use_emb = w + 7 * R;
  uint64_t *anc = reinterpret_cast<uint64_t *>(w + 8 * R);
  int32_t *kvl = w + 10 * R, *row_start = kvl + batch, *n_nodes = row_start + batch;
  int r = 0;
  for (int b = 0; b < batch; ++b) {
    const int n = tree->n_nodes[b];
    const int32_t *par = tree->parents + (size_t)b * c.max_nodes;
    const int32_t *tok = tree->tokens + (size_t)b * c.max_nodes;
    const int L = kv_len ? kv_len[b] : 0;
    kvl[b] = L;
    row_start[b] = r;
    n_nodes[b] = n;
    for (int i = 0; i < n; ++i, ++r) {
      const int p = par[i];
      token[r] = tok[i];
      seq[r] = b;
      node[r] = i;
      parent[r] = p;
      depth[r] = i == 0 ? 0 : depth[row_start[b] + p] + 1;
      anc[r] = (i == 0 ? 0ull : anc[row_start[b] + p]) | (1ull << i);
      pos[r] = L + depth[r];
      slot[r] = L + i;
      use_emb[r] = (tree->use_embed && tree->use_embed[(size_t)b * c.max_nodes + i]) ? 1 : 0;
      if (use_emb[r]) token[r] = 0;
    }
  }
}

StepMeta device_meta(const specasr_ctx *ctx, char *ws, const WsLayout &L, int batch_cap,
                     const HostStep &hs) {
  const int R = batch_cap * ctx->cfg.max_nodes;
  const int32_t *w = reinterpret_cast<const int32_t *>(ws + L.meta);
  StepMeta m;
  m.token = w;
  m.seq = w + R;
  m.node = w + 2 * R;
  m.depth = w + 3 * R;
  m.pos = w + 4 * R;
  m.slot = w + 5 * R;
  m.parent = w + 6 * R;
  m.use_embed = w + 7 * R;
  m.anc = reinterpret_cast<const uint64_t *>(w + 8 * R);
  m.kv_len = w + 10 * R;
  m.row_start = m.kv_len + batch_cap;
  m.n_nodes = m.row_start + batch_cap;
  m.rows = hs.rows;
  m.batch = hs.batch;
  return m;
}

// Pinned staging buffers and events are created on first use, so that a context can be
// created -- and every host-side validation exercised -- on a machine without a GPU.
specasr_status ensure_staging(specasr_ctx *ctx) {
  if (ctx->staging_ready) return SPECASR_OK;
  const specasr_config &c = ctx->cfg;
  HIP_TRY(ctx, hipGetDevice(&ctx->device));
  const size_t mw = meta_words(c.max_batch * c.max_nodes, c.max_batch);
  for (int i = 0; i < kStagingSlots; ++i) {
    if (!ctx->stage[i].host) HIP_TRY(ctx, hipHostMalloc((void **)&ctx->stage[i].host, mw * 4, hipHostMallocDefault));
    if (!ctx->stage[i].done) HIP_TRY(ctx, hipEventCreateWithFlags(&ctx->stage[i].done, hipEventDisableTiming));
  }
  ctx->out_host_words = (size_t)c.max_batch * c.max_nodes * 2 + (size_t)c.max_batch * 2;
  if (!ctx->out_host) HIP_TRY(ctx, hipHostMalloc((void **)&ctx->out_host, ctx->out_host_words * 4, hipHostMallocDefault));
  ctx->staging_ready = true;
  return SPECASR_OK;
}

// Next staging slot, free for reuse (its previous copy has completed).
specasr_status next_slot(specasr_ctx *ctx, Staging **out) {
  specasr_status s = ensure_staging(ctx);
  if (s != SPECASR_OK) return s;
  Staging &sg = ctx->stage[ctx->next_stage];
  ctx->next_stage = (ctx->next_stage + 1) % kStagingSlots;
  if (sg.used) HIP_TRY(ctx, hipEventSynchronize(sg.done));
  *out = &sg;
  return SPECASR_OK;
}

// Copy the metadata block to the device through a pinned staging slot.
specasr_status upload_meta(specasr_ctx *ctx, const HostStep &hs, char *ws, const WsLayout &L,
                           hipStream_t st) {
  Staging *sp = nullptr;
  specasr_status rc = next_slot(ctx, &sp);
  if (rc != SPECASR_OK) return rc;
  Staging &s = *sp;
  memcpy(s.host, hs.words.data(), hs.words.size() * 4);
  HIP_TRY(ctx, hipMemcpyAsync(ws + L.meta, s.host, hs.words.size() * 4, hipMemcpyHostToDevice, st));
  HIP_TRY(ctx, hipEventRecord(s.done, st));
  s.used = true;
  return SPECASR_OK;
}

specasr_status check_ws(const specasr_ctx *ctx, const void *ws, size_t bytes, int batch) {
  if (!ws) return SPECASR_E_WORKSPACE;
  if (((uintptr_t)ws & 255u) != 0) return SPECASR_E_WORKSPACE;
  if (bytes < ws_layout(ctx->cfg, batch).total) return SPECASR_E_WORKSPACE;
  return SPECASR_OK;
}

// Steps 1-8 with the dtype-generic kernels.
void forward_generic(specasr_ctx *ctx, const StepMeta &m, const KvGeom &g, specasr_kv *kv,
                     const specasr_tree *tree, char *ws, const WsLayout &L, int32_t *argmax_dev,
                     float *logits_dev, hipStream_t st) {
  const ModelDims &md = ctx->md;
  const int dt = md.dtype, d = md.d_model, F = md.d_ffn, V = md.vocab;
  const int dq = md.n_heads * md.head_dim, dkv = md.n_kv_heads * md.head_dim, R = m.rows;
  float *x = (float *)(ws + L.x), *h = (float *)(ws + L.h), *q = (float *)(ws + L.q);
  float *k = (float *)(ws + L.k), *v = (float *)(ws + L.v), *att = (float *)(ws + L.att);
  float *gu = (float *)(ws + L.gu), *t = (float *)(ws + L.t), *lg = (float *)(ws + L.logits);
  float2 *cs = (float2 *)(ws + L.rope);

  launch_rope_table(m, md.head_dim, md.rope_theta, cs, st);
  launch_embed(m, dt, ctx->w.tok_embed, tree->input_embeds, ctx->cfg.max_nodes, d, x, st);
  for (int l = 0; l < md.n_layers; ++l) {
    const specasr_layer_weights &lw = ctx->layers[l];
    launch_rmsnorm(dt, x, lw.attn_norm, R, d, md.rms_eps, h, st);
    launch_linear(dt, lw.wq, dq, d, h, d, q, dq, R, false, st);
    launch_linear(dt, lw.wk, dkv, d, h, d, k, dkv, R, false, st);
    launch_linear(dt, lw.wv, dkv, d, h, d, v, dkv, R, false, st);
    launch_rope_kv(m, md, g, l, cs, q, k, v, kv->k, kv->v, st);
    launch_attention_generic(m, md, g, l, q, kv->k, kv->v, att, st);
    launch_linear(dt, lw.wo, d, dq, att, dq, x, d, R, true, st);
    launch_rmsnorm(dt, x, lw.ffn_norm, R, d, md.rms_eps, h, st);
    launch_linear(dt, lw.w_gate, F, d, h, d, gu, 2 * F, R, false, st);
    launch_linear(dt, lw.w_up, F, d, h, d, gu + F, 2 * F, R, false, st);
    launch_swiglu(gu, R, F, t, st);
    launch_linear(dt, lw.w_down, d, F, t, F, x, d, R, true, st);
  }
  launch_rmsnorm(dt, x, ctx->w.final_norm, R, d, md.rms_eps, h, st);
  launch_linear(dt, ctx->w.lm_head, V, d, h, d, lg, V, R, false, st);
  launch_argmax(m, lg, false, ctx->cfg.max_nodes, V, argmax_dev, st);
  if (logits_dev) launch_scatter_logits(m, lg, ctx->cfg.max_nodes, V, logits_dev, st);
}

specasr_status forward_common(specasr_ctx *ctx, specasr_kv *kv, const specasr_tree *tree,
                              int32_t *argmax_dev, float *logits_dev, char *ws,
                              const WsLayout &L, const HostStep &hs, hipStream_t st) {
  KvGeom g{kv->capacity, ctx->md.n_layers, ctx->md.n_kv_heads, ctx->md.head_dim};
  StepMeta m = device_meta(ctx, ws, L, hs.batch, hs);
  forward_generic(ctx, m, g, kv, tree, ws, L, argmax_dev, logits_dev, st);
  HIP_TRY(ctx, hipGetLastError());
  return SPECASR_OK;
}

specasr_status check_kv(const specasr_kv *kv) {
  if (!kv || !kv->k || !kv->v || !kv->kv_len) return SPECASR_E_NULL;
  if (kv->capacity < 1 || kv->batch < 1) return SPECASR_E_KV_OVERFLOW;
  return SPECASR_OK;
}

}  // namespace

extern "C" {

int32_t specasr_abi_version(void) { return 1; }

const char *specasr_strerror(specasr_status s) {
  switch (s) {
    case SPECASR_OK: return "ok";
    case SPECASR_E_NULL: return "a required pointer is NULL";
    case SPECASR_E_CONFIG: return "inconsistent or unsupported model configuration";
    case SPECASR_E_TREE: return "invalid draft tree (size, parent order or token id)";
    case SPECASR_E_KV_OVERFLOW: return "kv_len out of range or tree does not fit the KV cache";
    case SPECASR_E_WORKSPACE: return "workspace missing, misaligned or too small";
    case SPECASR_E_HIP: return "HIP runtime error";
    case SPECASR_E_UNSUPPORTED: return "request not supported by this build";
    case SPECASR_E_PATH: return "path is not a valid root path";
  }
  return "unknown status";
}

int32_t specasr_last_hip_error(const specasr_ctx *ctx) { return ctx ? ctx->last_hip : 0; }

specasr_status specasr_create(const specasr_config *cfg, const specasr_weights *weights,
                              specasr_ctx **out) {
  if (!cfg || !weights || !out) return SPECASR_E_NULL;
  *out = nullptr;
  const specasr_config &c = *cfg;
  if (c.n_layers < 1 || c.d_model < 8 || c.n_heads < 1 || c.n_kv_heads < 1 || c.head_dim < 8 ||
      c.d_ffn < 8 || c.vocab < 1)
    return SPECASR_E_CONFIG;
  if (c.n_heads % c.n_kv_heads != 0) return SPECASR_E_CONFIG;
  if (c.d_model % 8 || c.d_ffn % 8 || c.head_dim % 8) return SPECASR_E_CONFIG;
  if (c.head_dim > 256 || 256 % c.head_dim != 0) return SPECASR_E_CONFIG;
  if (c.dtype != SPECASR_F32 && c.dtype != SPECASR_BF16) return SPECASR_E_CONFIG;
  if (c.max_nodes < 1 || c.max_nodes > SPECASR_MAX_NODES || c.max_batch < 1) return SPECASR_E_CONFIG;
  if (!(c.rms_eps >= 0.f) || !(c.rope_theta > 0.f)) return SPECASR_E_CONFIG;
  if (!weights->tok_embed || !weights->final_norm || !weights->lm_head || !weights->layers)
    return SPECASR_E_NULL;
  for (int l = 0; l < c.n_layers; ++l) {
    const specasr_layer_weights &lw = weights->layers[l];
    if (!lw.attn_norm || !lw.wq || !lw.wk || !lw.wv || !lw.wo || !lw.ffn_norm || !lw.w_gate ||
        !lw.w_up || !lw.w_down)
      return SPECASR_E_NULL;
  }
  specasr_ctx *ctx = new (std::nothrow) specasr_ctx();
  if (!ctx) return SPECASR_E_HIP;
  ctx->cfg = c;
  ctx->md = ModelDims{c.n_layers, c.d_model, c.n_heads, c.n_kv_heads, c.head_dim, c.d_ffn,
                      c.vocab, c.rms_eps, c.rope_theta, c.dtype};
  ctx->layers.assign(weights->layers, weights->layers + c.n_layers);
  ctx->w = *weights;
  ctx->w.layers = ctx->layers.data();
  *out = ctx;
  return SPECASR_OK;
}

void specasr_destroy(specasr_ctx *ctx) {
  if (!ctx) return;
  for (int i = 0; i < kStagingSlots; ++i) {
    if (ctx->stage[i].host) (void)hipHostFree(ctx->stage[i].host);
    if (ctx->stage[i].done) (void)hipEventDestroy(ctx->stage[i].done);
  }
  if (ctx->out_host) (void)hipHostFree(ctx->out_host);
  delete ctx;
}

size_t specasr_workspace_bytes(const specasr_ctx *ctx, int32_t batch) {
  if (!ctx || batch < 1 || batch > ctx->cfg.max_batch) return 0;
  return ws_layout(ctx->cfg, batch).total;
}

specasr_status specasr_tree_forward(specasr_ctx *ctx, specasr_kv *kv, const specasr_tree *tree,
                                    int32_t *argmax_dev, float *logits_dev, void *workspace,
                                    size_t workspace_bytes, void *stream) {
  if (!ctx || !argmax_dev) return SPECASR_E_NULL;
  specasr_status s = check_kv(kv);
  if (s != SPECASR_OK) return s;
  s = validate_tree(ctx, tree, kv->batch, kv->kv_len, kv->capacity, true);
  if (s != SPECASR_OK) return s;
  s = check_ws(ctx, workspace, workspace_bytes, kv->batch);
  if (s != SPECASR_OK) return s;
  hipStream_t st = (hipStream_t)stream;
  char *ws = (char *)workspace;
  const WsLayout L = ws_layout(ctx->cfg, kv->batch);
  HostStep hs;
  build_step(ctx, tree, kv->batch, kv->kv_len, &hs);
  s = upload_meta(ctx, hs, ws, L, st);
  if (s != SPECASR_OK) return s;
  return forward_common(ctx, kv, tree, argmax_dev, logits_dev, ws, L, hs, st);
}

specasr_status specasr_accept(specasr_ctx *ctx, const specasr_tree *tree, int32_t batch,
                              const int32_t *argmax_dev, int32_t *path_dev,
                              int32_t *accept_len_dev, int32_t *next_token_dev, void *workspace,
                              size_t workspace_bytes, void *stream) {
  if (!ctx || !argmax_dev || !path_dev || !accept_len_dev || !next_token_dev) return SPECASR_E_NULL;
  specasr_status s = validate_tree(ctx, tree, batch, nullptr, 0, false);
  if (s != SPECASR_OK) return s;
  s = check_ws(ctx, workspace, workspace_bytes, batch);
  if (s != SPECASR_OK) return s;
  hipStream_t st = (hipStream_t)stream;
  char *ws = (char *)workspace;
  const WsLayout L = ws_layout(ctx->cfg, batch);
  HostStep hs;
  build_step(ctx, tree, batch, nullptr, &hs);
  s = upload_meta(ctx, hs, ws, L, st);
  if (s != SPECASR_OK) return s;
  StepMeta m = device_meta(ctx, ws, L, batch, hs);
  launch_accept(m, ctx->cfg.max_nodes, argmax_dev, path_dev, accept_len_dev, next_token_dev, st);
  HIP_TRY(ctx, hipGetLastError());
  return SPECASR_OK;
}

specasr_status specasr_accept_from_logits(specasr_ctx *ctx, const specasr_tree *tree,
                                          int32_t batch, const float *logits_dev,
                                          int32_t *argmax_dev, int32_t *path_dev,
                                          int32_t *accept_len_dev, int32_t *next_token_dev,
                                          void *workspace, size_t workspace_bytes, void *stream) {
  if (!ctx || !logits_dev || !argmax_dev || !path_dev || !accept_len_dev || !next_token_dev)
    return SPECASR_E_NULL;
  specasr_status s = validate_tree(ctx, tree, batch, nullptr, 0, false);
  if (s != SPECASR_OK) return s;
  s = check_ws(ctx, workspace, workspace_bytes, batch);
  if (s != SPECASR_OK) return s;
  hipStream_t st = (hipStream_t)stream;
  char *ws = (char *)workspace;
  const WsLayout L = ws_layout(ctx->cfg, batch);
  HostStep hs;
  build_step(ctx, tree, batch, nullptr, &hs);
  s = upload_meta(ctx, hs, ws, L, st);
  if (s != SPECASR_OK) return s;
  StepMeta m = device_meta(ctx, ws, L, batch, hs);
  launch_argmax(m, logits_dev, true, ctx->cfg.max_nodes, ctx->cfg.vocab, argmax_dev, st);
  launch_accept(m, ctx->cfg.max_nodes, argmax_dev, path_dev, accept_len_dev, next_token_dev, st);
  HIP_TRY(ctx, hipGetLastError());
  return SPECASR_OK;
}

specasr_status specasr_commit(specasr_ctx *ctx, specasr_kv *kv, const int32_t *n_nodes,
                              const int32_t *path, const int32_t *accept_len, void *workspace,
                              size_t workspace_bytes, void *stream) {
  if (!ctx || !n_nodes || !path || !accept_len) return SPECASR_E_NULL;
  specasr_status s = check_kv(kv);
  if (s != SPECASR_OK) return s;
  const specasr_config &c = ctx->cfg;
  const int B = kv->batch;
  if (B > c.max_batch) return SPECASR_E_TREE;
  for (int b = 0; b < B; ++b) {
    const int n = n_nodes[b], len = accept_len[b];
    if (n < 1 || n > c.max_nodes) return SPECASR_E_TREE;
    if (kv->kv_len[b] < 0 || (int64_t)kv->kv_len[b] + n > kv->capacity) return SPECASR_E_KV_OVERFLOW;
    if (len < 1 || len > n) return SPECASR_E_PATH;
    const int32_t *p = path + (size_t)b * c.max_nodes;
    if (p[0] != 0) return SPECASR_E_PATH;
    for (int k = 1; k < len; ++k)
      if (p[k] <= p[k - 1] || p[k] >= n) return SPECASR_E_PATH;
  }
  s = check_ws(ctx, workspace, workspace_bytes, B);
  if (s != SPECASR_OK) return s;
  hipStream_t st = (hipStream_t)stream;
  char *ws = (char *)workspace;
  const WsLayout L = ws_layout(c, B);
  // stage [kv_len | accept_len | path] in the metadata region
  Staging *sgp = nullptr;
  s = next_slot(ctx, &sgp);
  if (s != SPECASR_OK) return s;
  Staging &sg = *sgp;
  int32_t *hw = sg.host;
  for (int b = 0; b < B; ++b) {
    hw[b] = kv->kv_len[b];
    hw[B + b] = accept_len[b];
    for (int k = 0; k < c.max_nodes; ++k)
      hw[2 * B + (size_t)b * c.max_nodes + k] = k < accept_len[b] ? path[(size_t)b * c.max_nodes + k] : -1;
  }
  const size_t words = 2 * (size_t)B + (size_t)B * c.max_nodes;
  int32_t *dw = reinterpret_cast<int32_t *>(ws + L.meta);
  HIP_TRY(ctx, hipMemcpyAsync(dw, hw, words * 4, hipMemcpyHostToDevice, st));
  HIP_TRY(ctx, hipEventRecord(sg.done, st));
  sg.used = true;
  KvGeom g{kv->capacity, c.n_layers, c.n_kv_heads, c.head_dim};
  launch_compact(c.dtype, g, B, c.max_nodes, dw, dw + 2 * B, dw + B, kv->k, kv->v, st);
  HIP_TRY(ctx, hipGetLastError());
  for (int b = 0; b < B; ++b) kv->kv_len[b] += accept_len[b];
  return SPECASR_OK;
}

specasr_status specasr_verify_tree(specasr_ctx *ctx, specasr_kv *kv, const specasr_tree *tree,
                                   specasr_out *out, void *workspace, size_t workspace_bytes,
                                   void *stream) {
  if (!ctx || !out || !out->argmax || !out->path || !out->accept_len || !out->next_token)
    return SPECASR_E_NULL;
  specasr_status s = check_kv(kv);
  if (s != SPECASR_OK) return s;
  s = validate_tree(ctx, tree, kv->batch, kv->kv_len, kv->capacity, true);
  if (s != SPECASR_OK) return s;
  s = check_ws(ctx, workspace, workspace_bytes, kv->batch);
  if (s != SPECASR_OK) return s;
  const specasr_config &c = ctx->cfg;
  const int B = kv->batch;
  hipStream_t st = (hipStream_t)stream;
  char *ws = (char *)workspace;
  const WsLayout L = ws_layout(c, B);
  HostStep hs;
  build_step(ctx, tree, B, kv->kv_len, &hs);
  s = upload_meta(ctx, hs, ws, L, st);
  if (s != SPECASR_OK) return s;
  int32_t *o = reinterpret_cast<int32_t *>(ws + L.outs);
  const size_t BN = (size_t)B * c.max_nodes;
  int32_t *argmax_dev = o, *path_dev = o + BN, *len_dev = o + 2 * BN, *next_dev = len_dev + B;
  s = forward_common(ctx, kv, tree, argmax_dev, out->logits, ws, L, hs, st);
  if (s != SPECASR_OK) return s;
  StepMeta m = device_meta(ctx, ws, L, B, hs);
  KvGeom g{kv->capacity, c.n_layers, c.n_kv_heads, c.head_dim};
  launch_accept(m, c.max_nodes, argmax_dev, path_dev, len_dev, next_dev, st);
  launch_compact(c.dtype, g, B, c.max_nodes, m.kv_len, path_dev, len_dev, kv->k, kv->v, st);
  HIP_TRY(ctx, hipGetLastError());
  const size_t words = 2 * BN + 2 * (size_t)B;
  HIP_TRY(ctx, hipMemcpyAsync(ctx->out_host, o, words * 4, hipMemcpyDeviceToHost, st));
  HIP_TRY(ctx, hipStreamSynchronize(st));
  const int32_t *h = ctx->out_host;
  for (int b = 0; b < B; ++b) {
    const int n = tree->n_nodes[b];
    for (int i = 0; i < c.max_nodes; ++i) {
      out->argmax[(size_t)b * c.max_nodes + i] = i < n ? h[(size_t)b * c.max_nodes + i] : -1;
      out->path[(size_t)b * c.max_nodes + i] = h[BN + (size_t)b * c.max_nodes + i];
    }
    out->accept_len[b] = h[2 * BN + b];
    out->next_token[b] = h[2 * BN + B + b];
    kv->kv_len[b] += out->accept_len[b];
  }
  return SPECASR_OK;
}

}  // extern "C"
