// C ABI and host dispatcher of the tree-verification library (see include/specasr.h).
// Validates on the host, stages the tree metadata through pinned memory, enqueues the
// stages on the caller's stream.
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>
#include <algorithm>
#include <chrono>
#include <mutex>
#include <vector>

#include "../../include/specasr.h"
#include "../../include/specasr_profile.h"
#include "kernels.h"
#include "kernels_mfma.h"

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
  size_t meta, outs, rope, x, h, q, k, v, att, gu, t, logits, top2_v, top2_i, total;
  size_t hb, attb, tb, part, ssq, blk_val, blk_idx;  // bf16 activations and split-k partial sums (MFMA path)
  size_t qb, attn_o, attn_ml;                   // MFMA attention: bf16 queries, per-chunk partial outputs
  size_t meta_words;
};

}  // namespace

// Packed (MFMA-tiled) weights of one decoder layer: q|k|v and gate|up are concatenated
// band-aligned so that each pair is one GEMM.
struct PackedLayer {
  PackedMatrix qkv, o, gu, down;
};

constexpr int kMaxLanes = 4;  // streams a multi-group call is spread over (lane 0 = the caller's)

// Development aids: environment variables that specasr_create reads ONCE into the context (no
// call reads the environment afterwards).  A deployment sets none of them.
struct Tuning {
  int lanes = kMaxLanes;                     // SPECASR_LANES: streams for multi-group calls, 1..4
  int gemm_splits[5] = {0, 0, 0, 0, 0};      // SPECASR_GEMM_SPLITS "qkv,o,gate_up,down,lm_head": k-splits of the skinny GEMMs (0: planner)
  int wide_splits[5] = {0, 0, 0, 0, 0};      // SPECASR_WIDE_SPLITS: the same for the tiled GEMM of wide passes
  int attn_chunk = 0;                        // SPECASR_ATTN_CHUNK: lower bound of the attention key chunk
  bool debug = false;                        // SPECASR_DEBUG: print kernel plans and host timings to stderr
  void read_env() {
    if (const char *e = getenv("SPECASR_LANES")) { const int v = atoi(e); lanes = v < 1 ? 1 : v > kMaxLanes ? kMaxLanes : v; }
    if (const char *e = getenv("SPECASR_GEMM_SPLITS")) sscanf(e, "%d,%d,%d,%d,%d", &gemm_splits[0], &gemm_splits[1], &gemm_splits[2], &gemm_splits[3], &gemm_splits[4]);
    if (const char *e = getenv("SPECASR_WIDE_SPLITS")) sscanf(e, "%d,%d,%d,%d,%d", &wide_splits[0], &wide_splits[1], &wide_splits[2], &wide_splits[3], &wide_splits[4]);
    if (const char *e = getenv("SPECASR_ATTN_CHUNK")) attn_chunk = atoi(e);
    debug = getenv("SPECASR_DEBUG") != nullptr;
  }
};

struct specasr_ctx {
  bool fast = false;  // bf16 MFMA path available (weights repacked)
  std::vector<PackedLayer> packed;
  PackedMatrix lm_head;
  std::vector<void *> owned;  // device allocations made by create
  int col_k = 0, col_v = 0, col_up = 0;  // column offsets inside the concatenated outputs
  size_t part_floats = 0;
  size_t wide_part_floats = 0;  // partial-sum buffer of a wide prefill pass, in floats (0: no wide path)
  // stage profiling (benchmark aid)
  int prof_stage = -1;
  int prof_mode = 1;         // 1: every launch of the stage, 2: only launches of the wide (prefill) kernel
  int64_t prof_rows = 0;     // activation rows summed over the timed launches
  std::vector<hipEvent_t> prof_ev;  // pairs
  size_t prof_used = 0;             // events recorded and not yet accumulated
  double prof_ms = 0.0;
  int64_t prof_launches = 0, prof_calls = 0;  // per-row-count-independent bound of the partial-sum buffer, in floats per row
  Tuning tune;
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
  int n_cu = 256;  // compute units = workgroups of the persistent-style GEMM grid
  bool staging_ready = false;
  // second lane for calls that run as several sequence groups: groups alternate between the
  // caller's stream and this one, so one group's latency-bound kernels overlap the other's GEMMs
  // prefill pipeline: per-layer events, two sets used alternately by consecutive chunks
  std::vector<hipEvent_t> layer_ev[2];
  hipStream_t lane_stream[kMaxLanes - 1] = {};
  hipEvent_t ev_fork = nullptr, ev_join[kMaxLanes - 1] = {};
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

constexpr size_t meta_words(int rows_max, int batch) {
  // token, seq, node, depth, pos, slot, parent, use_embed: 8 words per row; anc: 2 words per row;
  // kv_len, row_start, n_nodes: 3 words per sequence
  return (size_t)rows_max * 10 + (size_t)batch * 3;
}

inline int pad32(int v) { return (v + 31) / 32 * 32; }

// Chooses the k-split S of one skinny GEMM (workgroup g takes chunk g % S and every (P/S)-th
// band).  Cost model fitted to measurements on MI355X, in microseconds per wavefront: per weight
// tile streamed, per band (cross-wavefront reduction and partial write) and per k-step of
// activations loaded into registers -- 0.33 / 0.45 / 0.34 with one node group, 0.23 / 1.49 / 0.22
// with two (twice the accumulators to sum and store per band).  The slice of a wavefront must
// fit its ring.
GemmPlan plan_gemm(int n_bands, int ksteps, int nb, int n_cu) {
  GemmPlan best;
  double best_cost = 1e300;
  const int lw_max = nb == 1 ? 16 : 8;
  for (int S = 1; S <= 64; S *= 2) {
    if (n_cu % S) break;
    const int chunk = (ksteps + S - 1) / S;
    const int len = (chunk + 7) / 8;  // k-steps of the longest wavefront slice
    if (len > lw_max) continue;
    const int units = (n_bands + n_cu / S - 1) / (n_cu / S);
    const double cost = nb == 1 ? 0.33 * units * len + 0.45 * units + 0.34 * len
                                : 0.23 * units * len + 1.49 * units + 0.22 * len;
    if (cost < best_cost) {
      best_cost = cost;
      best.n_splits = S;
      best.lw = nb == 1 ? (len <= 4 ? 4 : len <= 8 ? 8 : len <= 12 ? 12 : 16) : (len <= 4 ? 4 : 8);
      best.grid = n_cu;
    }
  }
  return best;
}

WsLayout ws_layout(const specasr_ctx *ctx, int batch);

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
  L.top2_v = take(R * (size_t)top2_blocks(c.vocab) * 3 * 4);
  L.top2_i = take(R * (size_t)top2_blocks(c.vocab) * 2 * 4);
  L.total = off;
  return L;
}

// Workspace of a context: the generic regions plus, when the MFMA path exists, its bf16
// activation buffers and the split-k partial-sum buffer.
WsLayout ws_layout(const specasr_ctx *ctx, int batch) {
  const specasr_config &c = ctx->cfg;
  WsLayout L = ws_layout(c, batch);
  if (!ctx->fast) return L;
  const size_t R = (size_t)batch * c.max_nodes;
  const size_t dq = (size_t)c.n_heads * c.head_dim;
  size_t off = L.total;
  auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, 256); return o; };
  // packed activation buffers: hi and lo plane, each [k/16][node groups][64 lanes][8] for <= 64 rows
  L.hb = take(2 * 64 * (size_t)c.d_model * 2);
  L.attb = take(2 * 64 * dq * 2);
  L.tb = take(2 * 64 * (size_t)c.d_ffn * 2);
  L.part = take(64 * ctx->part_floats * 4);  // [split][band][rows padded to 32 or 64][32]
  L.ssq = take(64 * (size_t)residual_slabs(c.d_model) * 4);
  const size_t nblk = (size_t)logits_argmax_blocks(c.vocab);
  L.blk_val = take(R * nblk * 4);
  L.blk_idx = take(R * nblk * 4);
  L.qb = take(2 * R * dq * 2);
  const size_t mc = (size_t)tree_attention_max_chunks(c.n_kv_heads);
  L.attn_o = take(mc * R * dq * 4);
  L.attn_ml = take(mc * R * c.n_heads * 2 * 4);
  L.total = off;
  return L;
}

// A wide prefill pass takes up to kWideSeqs pieces of max_nodes consecutive positions of ONE
// sequence at once (each piece is a chain "tree" with its own kv_len on the shared cache), so
// that the projections become GEMMs over hundreds of rows.  Its buffers follow the lanes'.
constexpr int kWideSeqs = 16;

inline int wide_seqs(int batch) { return batch > kWideSeqs ? batch : kWideSeqs; }

WsLayout ws_layout_wide(const specasr_ctx *ctx, int batch) {
  const specasr_config &c = ctx->cfg;
  WsLayout L{};
  if (!ctx->fast || ctx->wide_part_floats == 0) return L;
  const size_t R = (size_t)wide_seqs(batch) * c.max_nodes, Rp = (size_t)wide_row_groups((int)R) * 32;
  const size_t dq = (size_t)c.n_heads * c.head_dim;
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, 256); return o; };
  L.meta_words = meta_words((int)R, wide_seqs(batch));
  L.meta = take(L.meta_words * 4);
  L.rope = take(R * (c.head_dim / 2) * sizeof(float2));
  L.x = take(R * c.d_model * 4);
  L.hb = take(2 * Rp * (size_t)c.d_model * 2);
  L.attb = take(2 * Rp * dq * 2);
  L.tb = take(2 * Rp * (size_t)c.d_ffn * 2);
  L.part = take(ctx->wide_part_floats * 4);
  L.ssq = take(R * (size_t)residual_slabs(c.d_model) * 4);
  L.qb = take(2 * R * dq * 2);
  // a pass has >= 2 pieces, so the key chunks of the attention number at most 128 / n_kv_heads + 1
  const size_t mc = (size_t)128 / c.n_kv_heads + 2;
  L.attn_o = take(mc * R * dq * 4);
  L.attn_ml = take(mc * R * c.n_heads * 2 * 4);
  // read-out of a wide verify / draft forward (a prefill pass has none)
  const size_t nblk = (size_t)logits_argmax_blocks(c.vocab);
  L.blk_val = take(R * nblk * 4);
  L.blk_idx = take(R * nblk * 4);
  L.top2_v = take(R * (size_t)top2_blocks(c.vocab) * 3 * 4);
  L.top2_i = take(R * (size_t)top2_blocks(c.vocab) * 2 * 4);
  L.outs = take(R * 4);  // argmax of a prefill pass, [piece][max_nodes]
  L.total = off;
  return L;
}

// Host-side view of one call: validated and flattened tree metadata.
struct HostStep {
  int rows = 0, batch = 0;
  int max_total_keys = 0;  // max over sequences of kv_len + n_nodes
  int max_seq_nodes = 0;
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
    if (L + n > hs->max_total_keys) hs->max_total_keys = L + n;
    if (n > hs->max_seq_nodes) hs->max_seq_nodes = n;
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
  const size_t R_host = (size_t)hs.batch * ctx->cfg.max_nodes;  // layout of hs.words
  m.kv_len0 = hs.words[10 * R_host];
  m.n_nodes0 = hs.words[10 * R_host + 2 * (size_t)hs.batch];
  return m;
}

// Pinned staging buffers and events are created on first use, so that a context can be
// created -- and every host-side validation exercised -- on a machine without a GPU.
specasr_status ensure_staging(specasr_ctx *ctx) {
  if (ctx->staging_ready) return SPECASR_OK;
  const specasr_config &c = ctx->cfg;
  HIP_TRY(ctx, hipGetDevice(&ctx->device));
  const int seqs_max = c.max_batch > kWideSeqs ? c.max_batch : kWideSeqs;
  const size_t mw = meta_words(seqs_max * c.max_nodes, seqs_max);
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

// A call that can fall into several sequence groups gets one workspace per lane (everything but the
// result block, which the lanes share).  Measured on config 4 (16 utterances, 8 groups): 13.8 ms
// with one lane, 10.6 with two, 9.0 with three or four (development aid: Tuning::lanes).
int ws_lanes(const specasr_ctx *ctx, int batch) {
  if (!ctx->fast) return 1;
  const int want = ctx->tune.lanes;
  if (want == 1) return 1;
  const int groups_max = (int)(((size_t)batch * ctx->cfg.max_nodes + 63) / 64);  // groups at full trees
  const int n = groups_max < want ? groups_max : want;
  return n < 2 ? 2 : n;  // two lanes at least: consecutive prefill chunks of one sequence overlap
}

specasr_status check_ws(const specasr_ctx *ctx, const void *ws, size_t bytes, int batch) {
  if (!ws) return SPECASR_E_WORKSPACE;
  if (((uintptr_t)ws & 255u) != 0) return SPECASR_E_WORKSPACE;
  if (bytes < ws_layout(ctx, batch).total * ws_lanes(ctx, batch) + ws_layout_wide(ctx, batch).total) return SPECASR_E_WORKSPACE;
  return SPECASR_OK;
}

// Distributes the sequence groups of one call over the lanes.  Lane 0 is the caller's stream;
// lane 1 (own stream, default priority) starts after everything already enqueued on the caller's
// stream and is joined back into it at the end, so the call stays asynchronous on one stream
// from the caller's point of view.
struct Lanes {
  specasr_ctx *ctx;
  hipStream_t st;
  char *ws;
  size_t lane_bytes;
  int n = 1;

  specasr_status begin(size_t n_groups, int batch) {
    n = ws_lanes(ctx, batch);
    if ((size_t)n > n_groups) n = (int)n_groups;
    if (n <= 1) { n = 1; return SPECASR_OK; }
    if (!ctx->ev_fork) HIP_TRY(ctx, hipEventCreateWithFlags(&ctx->ev_fork, hipEventDisableTiming));
    HIP_TRY(ctx, hipEventRecord(ctx->ev_fork, st));
    for (int l = 1; l < n; ++l) {
      if (!ctx->lane_stream[l - 1]) {
        HIP_TRY(ctx, hipStreamCreateWithFlags(&ctx->lane_stream[l - 1], hipStreamNonBlocking));
        HIP_TRY(ctx, hipEventCreateWithFlags(&ctx->ev_join[l - 1], hipEventDisableTiming));
      }
      HIP_TRY(ctx, hipStreamWaitEvent(ctx->lane_stream[l - 1], ctx->ev_fork, 0));
    }
    return SPECASR_OK;
  }
  hipStream_t stream(size_t gi) const { const int l = (int)(gi % n); return l ? ctx->lane_stream[l - 1] : st; }
  char *wsp(size_t gi) const { return ws + (gi % n) * lane_bytes; }
  specasr_status end() {
    for (int l = 1; l < n; ++l) {
      HIP_TRY(ctx, hipEventRecord(ctx->ev_join[l - 1], ctx->lane_stream[l - 1]));
      HIP_TRY(ctx, hipStreamWaitEvent(st, ctx->ev_join[l - 1], 0));
    }
    return SPECASR_OK;
  }
};

// What a forward leaves behind (device pointers in [batch][max_nodes] layout, already offset to
// the first sequence of the call or group).  Either argmax, or the draft-side read-out top2 +
// prob (then argmax is optional); logits always optional.
struct ReadOut {
  int32_t *argmax = nullptr;
  float *logits = nullptr;
  int32_t *top2 = nullptr;
  float *prob = nullptr;
  // Read-out only for rows >= first_row (at most 64 of them): a prefill pass over several pieces
  // of one sequence wants the token after its last position, not a vocabulary row per position.
  int first_row = 0;
  // nothing requested: the forward only fills the cache (all but the last pass of a prefill)
  bool none() const { return !argmax && !logits && !top2; }
};

// Steps 1-8 with the dtype-generic kernels.
void forward_generic(specasr_ctx *ctx, const StepMeta &m, const KvGeom &g, specasr_kv *kv,
                     const specasr_tree *tree, char *ws, const WsLayout &L, const ReadOut &ro,
                     hipStream_t st) {
  int32_t *argmax_dev = ro.argmax;
  float *logits_dev = ro.logits;
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
  if (ro.none()) return;
  launch_rmsnorm(dt, x, ctx->w.final_norm, R, d, md.rms_eps, h, st);
  launch_linear(dt, ctx->w.lm_head, V, d, h, d, lg, V, R, false, st);
  if (ro.top2)
    launch_top2(m, lg, false, 0, 0, RowNorm{nullptr, 0, 0, 0.f}, V, ctx->cfg.max_nodes, nullptr,
                (float *)(ws + L.top2_v), (int *)(ws + L.top2_i), ro.top2, ro.prob, argmax_dev, st);
  else
    launch_argmax(m, lg, false, ctx->cfg.max_nodes, V, argmax_dev, st);
  if (logits_dev) launch_scatter_logits(m, lg, ctx->cfg.max_nodes, V, logits_dev, st);
}

constexpr size_t kProfPairs = 256;

// Adds the elapsed time of every recorded event pair to the totals (waits for them).
specasr_status prof_drain(specasr_ctx *ctx) {
  for (size_t i = 0; i + 1 < ctx->prof_used; i += 2) {
    HIP_TRY(ctx, hipEventSynchronize(ctx->prof_ev[i + 1]));
    float ms = 0.f;
    HIP_TRY(ctx, hipEventElapsedTime(&ms, ctx->prof_ev[i], ctx->prof_ev[i + 1]));
    ctx->prof_ms += ms;
    ++ctx->prof_launches;
  }
  ctx->prof_used = 0;
  return SPECASR_OK;
}

// Launches one projection GEMM; brackets it with events when it is the profiled one.
void gemm_stage(specasr_ctx *ctx, int stage, bool profiled_layer, const PackedMatrix &W,
                const uint16_t *Xp, int rows, float *part, const GemmPlan &plan, hipStream_t st) {
  const bool prof = ctx->prof_stage == stage && profiled_layer && !ctx->prof_ev.empty() && (ctx->prof_mode != 2 || plan.wide);
  hipEvent_t ev0 = nullptr, ev1 = nullptr;
  if (prof) {
    if (ctx->prof_used + 2 > ctx->prof_ev.size()) (void)prof_drain(ctx);
    ev0 = ctx->prof_ev[ctx->prof_used];
    ev1 = ctx->prof_ev[ctx->prof_used + 1];
    ctx->prof_used += 2;
    ctx->prof_rows += rows;
  }
  if (plan.wide)
    launch_gemm_wide(W, Xp, rows, part, plan.n_splits, stage, st, ev0, ev1);
  else
    launch_gemm_skinny(W, Xp, rows, part, plan, stage, st, ev0, ev1);
}

// Ordering between two forwards that run on different streams and meet in the KV cache (chunk c+1
// of a prefill reads, layer by layer, the rows chunk c writes): `record[l]` is recorded once the
// K/V rows of layer l are in the cache, `wait[l]` is waited for before layer l's attention.
struct LayerSync {
  const hipEvent_t *wait = nullptr;
  const hipEvent_t *record = nullptr;
};

// Steps 1-8 with the bf16 MFMA kernels (rows <= 64: skinny GEMMs bound by the weight stream; more
// rows, a wide prefill pass: tiled GEMMs bound by the matrix cores).  Residual stream, norms, softmax and all
// accumulators stay fp32; only the MFMA operands (normalised activations, attention output,
// SwiGLU output) are rounded to bf16.
specasr_status forward_fast(specasr_ctx *ctx, const StepMeta &m, const KvGeom &g, specasr_kv *kv,
                            const specasr_tree *tree, char *ws, const WsLayout &L, const HostStep &hs,
                            const ReadOut &ro, const LayerSync &sync, hipStream_t st) {
  int32_t *argmax_dev = ro.argmax;
  float *logits_dev = ro.logits;
  const ModelDims &md = ctx->md;
  const int d = md.d_model, F = md.d_ffn, V = md.vocab, R = m.rows;
  const int dq = md.n_heads * md.head_dim;
  const bool wide = R > 64;
  const int nb = R <= 32 ? 1 : R <= 64 ? 2 : wide_row_groups(R);  // row groups of 32 in the packed planes
  float *x = (float *)(ws + L.x), *q = (float *)(ws + L.q), *att = (float *)(ws + L.att);
  float *part = (float *)(ws + L.part), *ssq = (float *)(ws + L.ssq);
  const RowNorm nrm{ssq, residual_slabs(d), d, md.rms_eps};
  uint16_t *hb = (uint16_t *)(ws + L.hb), *attb = (uint16_t *)(ws + L.attb), *tb = (uint16_t *)(ws + L.tb);
  // lo planes follow the hi planes: one plane holds k * 32 * nb elements
  uint16_t *hb_lo = hb + (size_t)d * 32 * nb, *attb_lo = attb + (size_t)dq * 32 * nb, *tb_lo = tb + (size_t)F * 32 * nb;
  float2 *cs = (float2 *)(ws + L.rope);
  uint16_t *qb = (uint16_t *)(ws + L.qb), *qb_lo = qb + (size_t)R * dq;
  const bool mfma_attn = tree_attention_supported(md.head_dim);
  const PackedLayer &p0 = ctx->packed[0];
  GemmPlan pl_qkv = plan_gemm(p0.qkv.n_bands, p0.qkv.ksteps, nb, ctx->n_cu);
  GemmPlan pl_o = plan_gemm(p0.o.n_bands, p0.o.ksteps, nb, ctx->n_cu);
  GemmPlan pl_gu = plan_gemm(p0.gu.n_bands, p0.gu.ksteps, nb, ctx->n_cu);
  GemmPlan pl_dn = plan_gemm(p0.down.n_bands, p0.down.ksteps, nb, ctx->n_cu);
  GemmPlan pl_lm = plan_gemm(ctx->lm_head.n_bands, ctx->lm_head.ksteps, nb, ctx->n_cu);
  if (wide) {
    GemmPlan *pls[5] = {&pl_qkv, &pl_o, &pl_gu, &pl_dn, &pl_lm};
    const PackedMatrix *pm[5] = {&p0.qkv, &p0.o, &p0.gu, &p0.down, &ctx->lm_head};
    for (int i = 0; i < 5; ++i) {
      pls[i]->wide = true;
      int S = wide_gemm_splits(pm[i]->n_bands, pm[i]->ksteps, R, ctx->n_cu);
      while (S > 1 && (size_t)S * pm[i]->ldo * part_rows_pad(R) > ctx->wide_part_floats) S /= 2;
      pls[i]->n_splits = S;
    }
    for (int i = 0; i < 5; ++i) {  // development aid: forced split counts
      const int v = ctx->tune.wide_splits[i];
      if (v >= 1 && v <= pm[i]->ksteps && (size_t)v * pm[i]->ldo * part_rows_pad(R) <= ctx->wide_part_floats)
        pls[i]->n_splits = v;
    }
  } else {
    GemmPlan *pls[5] = {&pl_qkv, &pl_o, &pl_gu, &pl_dn, &pl_lm};
    const PackedMatrix *pm[5] = {&p0.qkv, &p0.o, &p0.gu, &p0.down, &ctx->lm_head};
    for (int i = 0; i < 5; ++i) {  // development aid: forced split counts
      const int v = ctx->tune.gemm_splits[i];
      if (v < 1 || ctx->n_cu % v) continue;
      const int len = ((pm[i]->ksteps + v - 1) / v + 7) / 8;
      if (len > (nb == 1 ? 16 : 8) || (size_t)v * pm[i]->ldo > ctx->part_floats) continue;
      pls[i]->n_splits = v;
      pls[i]->lw = nb == 1 ? (len <= 4 ? 4 : len <= 8 ? 8 : len <= 12 ? 12 : 16) : (len <= 4 ? 4 : 8);
    }
  }
  if (ctx->tune.debug) {
    const GemmPlan *pls[5] = {&pl_qkv, &pl_o, &pl_gu, &pl_dn, &pl_lm};
    const char *nm[5] = {"qkv", "o", "gate_up", "down", "lm_head"};
    const PackedMatrix *pm[5] = {&p0.qkv, &p0.o, &p0.gu, &p0.down, &ctx->lm_head};
    for (int i = 0; i < 5; ++i)
      fprintf(stderr, "[specasr] %-8s bands=%d ksteps=%d rows=%d: %s splits=%d ring=%d grid=%d\n", nm[i],
              pm[i]->n_bands, pm[i]->ksteps, R, wide ? "wide" : "skinny", pls[i]->n_splits, pls[i]->lw, pls[i]->grid);
  }
  launch_rope_table(m, md.head_dim, md.rope_theta, cs, st);
  launch_embed(m, 1, ctx->w.tok_embed, tree->input_embeds, ctx->cfg.max_nodes, d, x, st);
  int pending = 0, pending_ld = 0;  // partial sums of the previous down projection, not yet added to x
  const int prof_layer = (int)(ctx->prof_calls++ % md.n_layers);
  for (int l = 0; l < md.n_layers; ++l) {
    const bool pl = l == prof_layer;
    const specasr_layer_weights &lw = ctx->layers[l];
    const PackedLayer &pk = ctx->packed[l];
    launch_residual_gain(x, part, pending, R, pending_ld, lw.attn_norm, d, hb, hb_lo, nb, ssq, st);
    gemm_stage(ctx, SPECASR_STAGE_QKV, pl, pk.qkv, hb, R, part, pl_qkv, st);
    if (mfma_attn) {
      launch_qkv_finish(m, md, g, l, part, pl_qkv.n_splits, pk.qkv.ldo, nrm, ctx->col_k, ctx->col_v, cs, nullptr, qb, qb_lo, kv->k, kv->v, st);
      if (sync.record) HIP_TRY(ctx, hipEventRecord(sync.record[l], st));
      if (sync.wait) HIP_TRY(ctx, hipStreamWaitEvent(st, sync.wait[l], 0));
      launch_tree_attention(m, md, g, l, hs.max_total_keys, hs.max_seq_nodes, qb, qb_lo, kv->k, kv->v,
                            (float *)(ws + L.attn_o), (float *)(ws + L.attn_ml), attb, attb_lo, nb, ctx->tune.attn_chunk, st);
    } else {
      launch_qkv_finish(m, md, g, l, part, pl_qkv.n_splits, pk.qkv.ldo, nrm, ctx->col_k, ctx->col_v, cs, q, nullptr, nullptr, kv->k, kv->v, st);
      if (sync.record) HIP_TRY(ctx, hipEventRecord(sync.record[l], st));
      if (sync.wait) HIP_TRY(ctx, hipStreamWaitEvent(st, sync.wait[l], 0));
      launch_attention_generic(m, md, g, l, q, kv->k, kv->v, att, st);
      launch_to_bf16(att, R, dq, attb, attb_lo, st);
    }
    gemm_stage(ctx, SPECASR_STAGE_O, pl, pk.o, attb, R, part, pl_o, st);
    launch_residual_gain(x, part, pl_o.n_splits, R, pk.o.ldo, lw.ffn_norm, d, hb, hb_lo, nb, ssq, st);
    gemm_stage(ctx, SPECASR_STAGE_GATE_UP, pl, pk.gu, hb, R, part, pl_gu, st);
    launch_swiglu_finish(part, pl_gu.n_splits, R, pk.gu.ldo, nrm, ctx->col_up, F, tb, tb_lo, nb, st);
    gemm_stage(ctx, SPECASR_STAGE_DOWN, pl, pk.down, tb, R, part, pl_dn, st);
    pending = pl_dn.n_splits;
    pending_ld = pk.down.ldo;
  }
  if (ro.none()) return SPECASR_OK;
  if (ro.first_row > 0) {
    // views of the last rows: residual, pending partial sums and row statistics start R0 rows in;
    // their planes are packed from row 0 again and go through the skinny LM head
    const int R0 = ro.first_row, Rs = R - R0, nbs = Rs <= 32 ? 1 : 2, n_slab = residual_slabs(d);
    StepMeta ms = m;
    ms.token += R0; ms.seq += R0; ms.node += R0; ms.depth += R0; ms.pos += R0; ms.slot += R0;
    ms.parent += R0; ms.use_embed += R0; ms.anc += R0;
    ms.rows = Rs;
    const RowNorm nrs{ssq + (size_t)R0 * n_slab, n_slab, d, md.rms_eps};
    launch_residual_gain(x + (size_t)R0 * d, part + (size_t)R0 * 32, pending, Rs, pending_ld, ctx->w.final_norm, d,
                         hb, hb + (size_t)d * 32 * nbs, nbs, ssq + (size_t)R0 * n_slab, st, part_rows_pad(R));
    const GemmPlan pls = plan_gemm(ctx->lm_head.n_bands, ctx->lm_head.ksteps, nbs, ctx->n_cu);
    gemm_stage(ctx, SPECASR_STAGE_LM_HEAD, true, ctx->lm_head, hb, Rs, part, pls, st);
    if (ro.top2)
      launch_top2(ms, part, true, pls.n_splits, ctx->lm_head.ldo, nrs, V, ctx->cfg.max_nodes, logits_dev,
                  (float *)(ws + L.top2_v), (int *)(ws + L.top2_i), ro.top2, ro.prob, argmax_dev, st);
    else
      launch_logits_argmax(ms, part, pls.n_splits, ctx->lm_head.ldo, nrs, V, ctx->cfg.max_nodes, logits_dev,
                           (float *)(ws + L.blk_val), (int *)(ws + L.blk_idx), argmax_dev, st);
    return SPECASR_OK;
  }
  launch_residual_gain(x, part, pending, R, pending_ld, ctx->w.final_norm, d, hb, hb_lo, nb, ssq, st);
  gemm_stage(ctx, SPECASR_STAGE_LM_HEAD, true, ctx->lm_head, hb, R, part, pl_lm, st);
  if (ro.top2)
    launch_top2(m, part, true, pl_lm.n_splits, ctx->lm_head.ldo, nrm, V, ctx->cfg.max_nodes, logits_dev,
                (float *)(ws + L.top2_v), (int *)(ws + L.top2_i), ro.top2, ro.prob, argmax_dev, st);
  else
    launch_logits_argmax(m, part, pl_lm.n_splits, ctx->lm_head.ldo, nrm, V, ctx->cfg.max_nodes, logits_dev,
                         (float *)(ws + L.blk_val), (int *)(ws + L.blk_idx), argmax_dev, st);
  return SPECASR_OK;
}

specasr_status forward_common(specasr_ctx *ctx, specasr_kv *kv, const specasr_tree *tree,
                              const ReadOut &ro, char *ws, const WsLayout &L, const HostStep &hs,
                              hipStream_t st, const LayerSync &sync = LayerSync(),
                              bool wide_ws = false, bool shared_cache = false) {
  KvGeom g{kv->capacity, ctx->md.n_layers, ctx->md.n_kv_heads, ctx->md.head_dim};
  g.shared_cache = shared_cache ? 1 : 0;
  StepMeta m = device_meta(ctx, ws, L, hs.batch, hs);
  if (ctx->fast && (m.rows <= 64 || wide_ws)) {
    const specasr_status s = forward_fast(ctx, m, g, kv, tree, ws, L, hs, ro, sync, st);
    if (s != SPECASR_OK) return s;
  } else
    forward_generic(ctx, m, g, kv, tree, ws, L, ro, st);
  HIP_TRY(ctx, hipGetLastError());
  return SPECASR_OK;
}

// A consecutive run of whole sequences of one call, with views of the caller's cache and trees
// that start at its first sequence.
struct SeqGroup {
  int s0 = 0;  // first sequence
  specasr_kv kv{};
  specasr_tree tree{};
};

// The MFMA kernels take at most 64 activation rows, so a call with more tree nodes in total is
// run as consecutive groups of whole sequences with <= 64 rows each (a tree has <= 64 nodes);
// the dtype-generic kernels take the whole call at once.
// Where the context has the wide buffers, a call with more than 64 rows is ONE group on the wide
// kernels instead: the weights are streamed once, not once per group (7B, 2 x 64 nodes: 6.8 ms
// against 8.5 in two groups).  SPECASR_FLAG_NO_WIDE creates a context without them.
std::vector<SeqGroup> split_call(const specasr_ctx *ctx, const specasr_kv *kv, const specasr_tree *tree,
                                 bool *wide) {
  const specasr_config &c = ctx->cfg;
  int total = 0;
  for (int b = 0; b < kv->batch; ++b) total += tree->n_nodes[b];
  *wide = ctx->fast && ctx->wide_part_floats > 0 && total > 64;
  const size_t esz = c.dtype == SPECASR_BF16 ? 2 : 4;
  const size_t seq_kv_bytes = (size_t)c.n_layers * c.n_kv_heads * (size_t)kv->capacity * c.head_dim * esz;
  std::vector<SeqGroup> out;
  int b = 0;
  while (b < kv->batch) {
    int e = b, rows = 0;
    while (e < kv->batch && (!ctx->fast || *wide || rows + tree->n_nodes[e] <= 64)) rows += tree->n_nodes[e++];
    SeqGroup g;
    g.s0 = b;
    g.kv.k = (char *)kv->k + (size_t)b * seq_kv_bytes;
    g.kv.v = (char *)kv->v + (size_t)b * seq_kv_bytes;
    g.kv.capacity = kv->capacity;
    g.kv.batch = e - b;
    g.kv.kv_len = kv->kv_len + b;
    g.tree.tokens = tree->tokens + (size_t)b * c.max_nodes;
    g.tree.parents = tree->parents + (size_t)b * c.max_nodes;
    g.tree.n_nodes = tree->n_nodes + b;
    g.tree.input_embeds = tree->input_embeds ? (const char *)tree->input_embeds + (size_t)b * c.max_nodes * c.d_model * esz : nullptr;
    g.tree.use_embed = tree->use_embed ? tree->use_embed + (size_t)b * c.max_nodes : nullptr;
    out.push_back(g);
    b = e;
  }
  return out;
}

// One-time repack of the bf16 weights into MFMA-tile order (values unchanged).  Allocates the
// packed copies; q|k|v and gate|up are concatenated, each part starting on a 32-row band.
specasr_status build_packed(specasr_ctx *ctx) {
  const specasr_config &c = ctx->cfg;
  const int d = c.d_model, F = c.d_ffn, dq = c.n_heads * c.head_dim, dkv = c.n_kv_heads * c.head_dim;
  HIP_TRY(ctx, gemm_skinny_set_lds_limit());
  HIP_TRY(ctx, tree_attention_set_lds_limit());
  {
    int dev = 0, cus = 0;
    HIP_TRY(ctx, hipGetDevice(&dev));
    HIP_TRY(ctx, hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
    if (cus >= 8) ctx->n_cu = cus;
  }
  auto alloc = [&](PackedMatrix &pm, int n_out_padded, int K) -> hipError_t {
    pm.n_bands = n_out_padded / 32;
    pm.ksteps = K / 16;
    pm.ldo = n_out_padded;
    hipError_t e = hipMalloc(&pm.data, (size_t)n_out_padded * K * 2);
    if (e == hipSuccess) ctx->owned.push_back(pm.data);
    return e;
  };
  ctx->col_k = pad32(dq);
  ctx->col_v = ctx->col_k + pad32(dkv);
  ctx->col_up = pad32(F);
  ctx->packed.resize(c.n_layers);
  hipStream_t st = nullptr;
  for (int l = 0; l < c.n_layers; ++l) {
    const specasr_layer_weights &lw = ctx->layers[l];
    PackedLayer &pk = ctx->packed[l];
    HIP_TRY(ctx, alloc(pk.qkv, ctx->col_v + pad32(dkv), d));
    launch_repack(lw.wq, dq, d, pk.qkv.data, 0, st);
    launch_repack(lw.wk, dkv, d, pk.qkv.data, ctx->col_k / 32, st);
    launch_repack(lw.wv, dkv, d, pk.qkv.data, ctx->col_v / 32, st);
    HIP_TRY(ctx, alloc(pk.o, pad32(d), dq));
    launch_repack(lw.wo, d, dq, pk.o.data, 0, st);
    HIP_TRY(ctx, alloc(pk.gu, 2 * pad32(F), d));
    launch_repack(lw.w_gate, F, d, pk.gu.data, 0, st);
    launch_repack(lw.w_up, F, d, pk.gu.data, ctx->col_up / 32, st);
    HIP_TRY(ctx, alloc(pk.down, pad32(d), F));
    launch_repack(lw.w_down, d, F, pk.down.data, 0, st);
    HIP_TRY(ctx, hipGetLastError());
  }
  HIP_TRY(ctx, alloc(ctx->lm_head, pad32(c.vocab), d));
  launch_repack(ctx->w.lm_head, c.vocab, d, ctx->lm_head.data, 0, st);
  HIP_TRY(ctx, hipGetLastError());
  HIP_TRY(ctx, hipStreamSynchronize(st));
  // bound of the partial-sum buffer: floats per activation row, over every GEMM and both widths
  size_t bound = 0;
  const PackedLayer &p0 = ctx->packed[0];
  const PackedMatrix *mats[5] = {&p0.qkv, &p0.o, &p0.gu, &p0.down, &ctx->lm_head};
  for (const PackedMatrix *pm : mats)
    for (int nb = 1; nb <= 2; ++nb) {
      const GemmPlan pl = plan_gemm(pm->n_bands, pm->ksteps, nb, ctx->n_cu);
      // the longest wavefront slice must fit the ring; otherwise this shape stays on the generic path
      if (((pm->ksteps + pl.n_splits - 1) / pl.n_splits + 7) / 8 > pl.lw) return SPECASR_E_UNSUPPORTED;
      const size_t need = (size_t)pl.n_splits * pm->ldo;
      if (need > bound) bound = need;
    }
  ctx->part_floats = bound;
  // wide passes: more than 64 rows at once -- prefill pieces or the trees of a batch (MFMA attention only)
  const bool wide_off = (c.flags & SPECASR_FLAG_NO_WIDE) != 0;
  if (tree_attention_supported(c.head_dim) && !wide_off) {
    size_t wb = 0;
    const int rows_max = wide_seqs(c.max_batch) * c.max_nodes;
    for (int rows = 64; rows < rows_max + 64; rows += 64) {  // splits and padding change only at multiples of 64
      for (const PackedMatrix *pm : mats) {
        const size_t need = (size_t)wide_gemm_splits(pm->n_bands, pm->ksteps, rows, ctx->n_cu) * pm->ldo * part_rows_pad(rows);
        if (need > wb) wb = need;
      }
    }
    // a pass of few short pieces (<= 64 rows in all) runs on the skinny kernels in the same buffers
    if (wb < 64 * bound) wb = 64 * bound;
    ctx->wide_part_floats = wb;
  }
  ctx->fast = true;
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

int32_t specasr_uses_mfma(const specasr_ctx *ctx, int32_t rows) {
  return (ctx && ctx->fast && rows >= 1) ? 1 : 0;
}

specasr_status specasr_profile_stage(specasr_ctx *ctx, int32_t stage, int32_t enable) {
  if (!ctx) return SPECASR_E_NULL;
  if (stage < SPECASR_STAGE_QKV || stage > SPECASR_STAGE_LM_HEAD) return SPECASR_E_UNSUPPORTED;
  if (!ctx->fast) return SPECASR_E_UNSUPPORTED;
  if (enable) {
    while (ctx->prof_ev.size() < 2 * kProfPairs) {
      hipEvent_t e;
      HIP_TRY(ctx, hipEventCreate(&e));
      ctx->prof_ev.push_back(e);
    }
    ctx->prof_stage = stage;
    ctx->prof_mode = enable == 2 ? 2 : 1;
    ctx->prof_used = 0;
    ctx->prof_ms = 0.0;
    ctx->prof_launches = 0;
    ctx->prof_rows = 0;
  } else {
    ctx->prof_stage = -1;
  }
  return SPECASR_OK;
}

specasr_status specasr_stage_time(specasr_ctx *ctx, double *total_ms, int64_t *launches,
                                  double *weight_bytes_per_launch) {
  if (!ctx || !total_ms || !launches || !weight_bytes_per_launch) return SPECASR_E_NULL;
  if (ctx->prof_stage < 0 || !ctx->fast) return SPECASR_E_UNSUPPORTED;
  specasr_status s = prof_drain(ctx);
  if (s != SPECASR_OK) return s;
  const specasr_config &c = ctx->cfg;
  const double d = c.d_model, dq = (double)c.n_heads * c.head_dim, dkv = (double)c.n_kv_heads * c.head_dim;
  const double elems[5] = {(dq + 2 * dkv) * d, d * dq, 2.0 * c.d_ffn * d, d * c.d_ffn, (double)c.vocab * d};
  *total_ms = ctx->prof_ms;
  *launches = ctx->prof_launches;
  *weight_bytes_per_launch = elems[ctx->prof_stage] * 2.0;
  return SPECASR_OK;
}

specasr_status specasr_read_ceiling(specasr_ctx *ctx, const void *buf_dev, size_t bytes, int32_t reps,
                                    void *stream, double *gb_per_s) {
  if (!ctx || !buf_dev || !gb_per_s) return SPECASR_E_NULL;
  if (bytes < (1u << 20) || reps < 1 || ((uintptr_t)buf_dev & 15u)) return SPECASR_E_UNSUPPORTED;
  hipStream_t st = (hipStream_t)stream;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  HIP_TRY(ctx, hipEventCreate(&e0));
  hipError_t err = hipEventCreate(&e1);
  // the probe never stores: its sink is only named in a branch that is never taken
  uint32_t *sink = (uint32_t *)const_cast<void *>(buf_dev);
  if (err == hipSuccess) {
    launch_read_probe(buf_dev, bytes, ctx->n_cu, sink, st);  // untimed first pass
    err = hipEventRecord(e0, st);
    for (int i = 0; i < reps && err == hipSuccess; ++i) launch_read_probe(buf_dev, bytes, ctx->n_cu, sink, st);
    if (err == hipSuccess) err = hipEventRecord(e1, st);
    if (err == hipSuccess) err = hipEventSynchronize(e1);
    float ms = 0.f;
    if (err == hipSuccess) err = hipEventElapsedTime(&ms, e0, e1);
    if (err == hipSuccess) err = hipGetLastError();
    if (err == hipSuccess) *gb_per_s = (double)(bytes / 16 * 16) * reps / (ms * 1e-3) / 1e9;
  }
  (void)hipEventDestroy(e0);
  if (e1) (void)hipEventDestroy(e1);
  HIP_TRY(ctx, err);
  return SPECASR_OK;
}

specasr_status specasr_stage_rows(specasr_ctx *ctx, int64_t *rows) {
  if (!ctx || !rows) return SPECASR_E_NULL;
  if (ctx->prof_stage < 0 || !ctx->fast) return SPECASR_E_UNSUPPORTED;
  specasr_status s = prof_drain(ctx);
  if (s != SPECASR_OK) return s;
  *rows = ctx->prof_rows;
  return SPECASR_OK;
}

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
  ctx->tune.read_env();
  ctx->layers.assign(weights->layers, weights->layers + c.n_layers);
  ctx->w = *weights;
  ctx->w.layers = ctx->layers.data();
  const bool want_fast = c.dtype == SPECASR_BF16 && !(c.flags & SPECASR_FLAG_GENERIC_KERNELS) &&
                         !(c.flags & SPECASR_FLAG_NO_REPACK) && c.d_model % 16 == 0 &&
                         c.d_ffn % 16 == 0 && (c.n_heads * c.head_dim) % 16 == 0;
  if (want_fast) {
    specasr_status rs = build_packed(ctx);
    if (rs == SPECASR_E_UNSUPPORTED) {
      for (void *p : ctx->owned) (void)hipFree(p);
      ctx->owned.clear();
      ctx->packed.clear();
      ctx->fast = false;
    } else if (rs != SPECASR_OK) {
      const int32_t he = ctx->last_hip;
      specasr_destroy(ctx);
      (void)he;
      return rs;
    }
  }
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
  for (void *p : ctx->owned) (void)hipFree(p);
  if (ctx->ev_fork) (void)hipEventDestroy(ctx->ev_fork);
  for (auto &set : ctx->layer_ev)
    for (hipEvent_t e : set) (void)hipEventDestroy(e);
  for (int l = 0; l < kMaxLanes - 1; ++l) {
    if (ctx->ev_join[l]) (void)hipEventDestroy(ctx->ev_join[l]);
    if (ctx->lane_stream[l]) (void)hipStreamDestroy(ctx->lane_stream[l]);
  }
  for (hipEvent_t e : ctx->prof_ev) (void)hipEventDestroy(e);
  delete ctx;
}

size_t specasr_workspace_bytes(const specasr_ctx *ctx, int32_t batch) {
  if (!ctx || batch < 1 || batch > ctx->cfg.max_batch) return 0;
  return ws_layout(ctx, batch).total * ws_lanes(ctx, batch) + ws_layout_wide(ctx, batch).total;
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
  const WsLayout L = ws_layout(ctx, kv->batch);
  const size_t MN = (size_t)ctx->cfg.max_nodes;
  bool wide = false;
  std::vector<SeqGroup> groups = split_call(ctx, kv, tree, &wide);
  const WsLayout Lg = wide ? ws_layout_wide(ctx, kv->batch) : L;  // a wide call is one group in the wide buffers
  char *wide_ws = ws + L.total * ws_lanes(ctx, kv->batch);
  Lanes lanes{ctx, st, ws, L.total};
  s = lanes.begin(groups.size(), kv->batch);
  if (s != SPECASR_OK) return s;
  for (size_t gi = 0; gi < groups.size(); ++gi) {
    SeqGroup &grp = groups[gi];
    char *wl = wide ? wide_ws : lanes.wsp(gi);
    HostStep hs;
    build_step(ctx, &grp.tree, grp.kv.batch, grp.kv.kv_len, &hs);
    s = upload_meta(ctx, hs, wl, Lg, lanes.stream(gi));
    if (s != SPECASR_OK) return s;
    ReadOut ro;
    ro.argmax = argmax_dev + grp.s0 * MN;
    ro.logits = logits_dev ? logits_dev + grp.s0 * MN * ctx->cfg.vocab : nullptr;
    s = forward_common(ctx, &grp.kv, &grp.tree, ro, wl, Lg, hs, lanes.stream(gi), LayerSync(), wide);
    if (s != SPECASR_OK) return s;
  }
  return lanes.end();
}

specasr_status specasr_tree_forward_top2(specasr_ctx *ctx, specasr_kv *kv, const specasr_tree *tree,
                                         int32_t *top2_dev, float *top1_prob_dev, float *logits_dev,
                                         void *workspace, size_t workspace_bytes, void *stream) {
  if (!ctx || !top2_dev || !top1_prob_dev) return SPECASR_E_NULL;
  specasr_status s = check_kv(kv);
  if (s != SPECASR_OK) return s;
  s = validate_tree(ctx, tree, kv->batch, kv->kv_len, kv->capacity, true);
  if (s != SPECASR_OK) return s;
  s = check_ws(ctx, workspace, workspace_bytes, kv->batch);
  if (s != SPECASR_OK) return s;
  hipStream_t st = (hipStream_t)stream;
  char *ws = (char *)workspace;
  const WsLayout L = ws_layout(ctx, kv->batch);
  const size_t MN = (size_t)ctx->cfg.max_nodes;
  bool wide = false;
  std::vector<SeqGroup> groups = split_call(ctx, kv, tree, &wide);
  const WsLayout Lg = wide ? ws_layout_wide(ctx, kv->batch) : L;  // a wide call is one group in the wide buffers
  char *wide_ws = ws + L.total * ws_lanes(ctx, kv->batch);
  Lanes lanes{ctx, st, ws, L.total};
  s = lanes.begin(groups.size(), kv->batch);
  if (s != SPECASR_OK) return s;
  for (size_t gi = 0; gi < groups.size(); ++gi) {
    SeqGroup &grp = groups[gi];
    char *wl = wide ? wide_ws : lanes.wsp(gi);
    HostStep hs;
    build_step(ctx, &grp.tree, grp.kv.batch, grp.kv.kv_len, &hs);
    s = upload_meta(ctx, hs, wl, Lg, lanes.stream(gi));
    if (s != SPECASR_OK) return s;
    ReadOut ro;
    ro.top2 = top2_dev + grp.s0 * MN * 2;
    ro.prob = top1_prob_dev + grp.s0 * MN;
    ro.logits = logits_dev ? logits_dev + grp.s0 * MN * ctx->cfg.vocab : nullptr;
    s = forward_common(ctx, &grp.kv, &grp.tree, ro, wl, Lg, hs, lanes.stream(gi), LayerSync(), wide);
    if (s != SPECASR_OK) return s;
  }
  return lanes.end();
}

specasr_status specasr_prefill(specasr_ctx *ctx, specasr_kv *kv, const int32_t *tokens,
                               const void *input_embeds, const uint8_t *use_embed,
                               const int32_t *n_pos, int32_t max_pos, int32_t *next_token,
                               void *workspace, size_t workspace_bytes, void *stream) {
  if (!ctx || !n_pos || (!tokens && !input_embeds)) return SPECASR_E_NULL;
  if ((input_embeds == nullptr) != (use_embed == nullptr)) return SPECASR_E_NULL;
  specasr_status s = check_kv(kv);
  if (s != SPECASR_OK) return s;
  const specasr_config &c = ctx->cfg;
  const int B = kv->batch;
  if (B > c.max_batch || max_pos < 1) return SPECASR_E_TREE;
  for (int b = 0; b < B; ++b) {
    if (n_pos[b] < 0 || n_pos[b] > max_pos) return SPECASR_E_TREE;
    if (kv->kv_len[b] < 0 || (int64_t)kv->kv_len[b] + n_pos[b] > kv->capacity) return SPECASR_E_KV_OVERFLOW;
    for (int i = 0; i < n_pos[b]; ++i) {
      const size_t at = (size_t)b * max_pos + i;
      if (use_embed && use_embed[at]) continue;
      if (!tokens || tokens[at] < 0 || tokens[at] >= c.vocab) return SPECASR_E_TREE;
    }
  }
  s = check_ws(ctx, workspace, workspace_bytes, B);
  if (s != SPECASR_OK) return s;
  hipStream_t st = (hipStream_t)stream;
  char *ws = (char *)workspace;
  const WsLayout L = ws_layout(ctx, B);
  const size_t esz = c.dtype == SPECASR_BF16 ? 2 : 4;
  const size_t seq_kv_bytes = (size_t)c.n_layers * c.n_kv_heads * (size_t)kv->capacity * c.head_dim * esz;
  int32_t *argmax_dev = reinterpret_cast<int32_t *>(ws + L.outs);  // [batch][max_nodes], last chunk of each sequence
  std::vector<int32_t> chunk_tok(c.max_nodes), chain(c.max_nodes);
  for (int i = 0; i < c.max_nodes; ++i) chain[i] = i - 1;
  std::vector<int32_t> kv_len_now(kv->kv_len, kv->kv_len + B);
  // Work list.  Where the context has the wide buffers, a sequence that adds more than one chunk
  // is taken in passes of up to kWideSeqs pieces of max_nodes positions (projections as
  // matrix-core-bound GEMMs over hundreds of rows); the pass that holds the last position reads out
  // the token after it from its last piece only.  One more 128-row tile through every GEMM costs
  // less than a chunk of its own on the skinny kernels, which stream every weight once more
  // (measured on the 7B prefix of 810 positions: 24.9 against 27.8 ms).  Contexts without wide
  // buffers, and sequences that add a single chunk, take chunks on the skinny kernels.
  struct Item { int b, c0, n; bool wide; };
  std::vector<Item> items;
  const WsLayout LW = ws_layout_wide(ctx, B);
  bool any_wide = false;
  for (int b = 0; b < B; ++b) {
    int c0 = 0;
    if (LW.total > 0 && n_pos[b] > 0) {
      const int wide_total = n_pos[b] > c.max_nodes ? n_pos[b] : 0;
      while (c0 < wide_total) {
        const int n = std::min(wide_total - c0, kWideSeqs * c.max_nodes);
        items.push_back({b, c0, n, true});
        any_wide = true;
        c0 += n;
      }
    }
    for (; c0 < n_pos[b]; c0 += c.max_nodes) items.push_back({b, c0, std::min<int>(c.max_nodes, n_pos[b] - c0), false});
  }
  // Without wide passes, consecutive chunks alternate between two lanes.  Chunk c+1 needs, at layer
  // l, the K/V rows chunk c wrote at layer l and nothing else of it, so it runs one layer behind on
  // the other stream and its latency-bound kernels fall under the other chunk's GEMMs.
  Lanes lanes{ctx, st, ws, L.total};
  const bool pipelined = ctx->fast && !any_wide && items.size() > 1 && ws_lanes(ctx, B) >= 2;
  if (pipelined) {
    s = lanes.begin(2, B);
    if (s != SPECASR_OK) return s;
    lanes.n = 2;
    for (auto &set : ctx->layer_ev)
      while ((int)set.size() < c.n_layers) {
        hipEvent_t e;
        HIP_TRY(ctx, hipEventCreateWithFlags(&e, hipEventDisableTiming));
        set.push_back(e);
      }
  }
  char *wide_ws = ws + L.total * ws_lanes(ctx, B);
  std::vector<int32_t> wide_parents, wide_n, wide_kv;
  int prev_b = -1;
  for (size_t ci = 0; ci < items.size(); ++ci) {
    const Item &it = items[ci];
    const int b = it.b;
    const size_t at = (size_t)b * max_pos + it.c0;
    specasr_kv kvv{(char *)kv->k + (size_t)b * seq_kv_bytes, (char *)kv->v + (size_t)b * seq_kv_bytes,
                   kv->capacity, 1, &kv_len_now[b]};
    const void *emb = input_embeds ? (const char *)input_embeds + at * c.d_model * esz : nullptr;
    if (it.wide) {
      // piece j: positions c0 + j * max_nodes ..., a chain on top of kv_len + j * max_nodes cached
      // rows; only the last piece of a sequence can be shorter than max_nodes
      const int pieces = (it.n + c.max_nodes - 1) / c.max_nodes;
      wide_parents.resize((size_t)pieces * c.max_nodes);
      wide_n.assign(pieces, c.max_nodes);
      wide_n[pieces - 1] = it.n - (pieces - 1) * c.max_nodes;
      wide_kv.resize(pieces);
      std::vector<int32_t> toks((size_t)it.n, 0);
      for (int i = 0; i < pieces * c.max_nodes; ++i) wide_parents[i] = i % c.max_nodes - 1;
      if (tokens)
        for (int i = 0; i < it.n; ++i) toks[i] = tokens[at + i];
      for (int j = 0; j < pieces; ++j) wide_kv[j] = kv_len_now[b] + j * c.max_nodes;
      kvv.batch = pieces;
      kvv.kv_len = wide_kv.data();
      specasr_tree tv{toks.data(), wide_parents.data(), wide_n.data(), emb, use_embed ? use_embed + at : nullptr};
      HostStep hs;
      build_step(ctx, &tv, pieces, wide_kv.data(), &hs);
      s = upload_meta(ctx, hs, wide_ws, LW, st);
      if (s != SPECASR_OK) return s;
      ReadOut ro;
      const bool last = it.c0 + it.n == n_pos[b];
      if (last && next_token) {
        ro.argmax = reinterpret_cast<int32_t *>(wide_ws + LW.outs);
        ro.first_row = (pieces - 1) * c.max_nodes;
      }
      s = forward_common(ctx, &kvv, &tv, ro, wide_ws, LW, hs, st, LayerSync(), true, true);
      if (s != SPECASR_OK) return s;
      if (last && next_token) {  // into the per-sequence slot the final copies read
        HIP_TRY(ctx, hipMemcpyAsync(argmax_dev + (size_t)b * c.max_nodes, ro.argmax + (size_t)(pieces - 1) * c.max_nodes,
                                    (size_t)c.max_nodes * 4, hipMemcpyDeviceToDevice, st));
      }
    } else {
      const int32_t n = it.n;
      const bool last = it.c0 + n == n_pos[b];
      for (int i = 0; i < n; ++i) chunk_tok[i] = tokens ? tokens[at + i] : 0;
      specasr_tree tv{chunk_tok.data(), chain.data(), &n, emb, use_embed ? use_embed + at : nullptr};
      char *wl = pipelined ? lanes.wsp(ci) : ws;
      hipStream_t sl = pipelined ? lanes.stream(ci) : st;
      HostStep hs;
      build_step(ctx, &tv, 1, kvv.kv_len, &hs);
      s = upload_meta(ctx, hs, wl, L, sl);
      if (s != SPECASR_OK) return s;
      ReadOut ro;
      if (last && next_token) ro.argmax = argmax_dev + (size_t)b * c.max_nodes;
      LayerSync sync;
      if (pipelined) {
        sync.record = ctx->layer_ev[ci & 1].data();
        if (b == prev_b) sync.wait = ctx->layer_ev[(ci + 1) & 1].data();  // the previous chunk's set
      }
      s = forward_common(ctx, &kvv, &tv, ro, wl, L, hs, sl, sync);
      if (s != SPECASR_OK) return s;
    }
    kv_len_now[b] += it.n;  // a chain's rows already sit in slots kv_len .. kv_len+n-1, in order
    prev_b = b;
  }
  if (pipelined) {
    s = lanes.end();
    if (s != SPECASR_OK) return s;
  }
  if (next_token) {
    bool any_result = false;
    for (int b = 0; b < B; ++b) {
      next_token[b] = -1;
      if (n_pos[b] <= 0) continue;
      const int32_t n_last = (n_pos[b] - 1) % c.max_nodes + 1;
      s = ensure_staging(ctx);
      if (s != SPECASR_OK) return s;
      HIP_TRY(ctx, hipMemcpyAsync(ctx->out_host + b, argmax_dev + (size_t)b * c.max_nodes + (n_last - 1), 4,
                                  hipMemcpyDeviceToHost, st));
      any_result = true;
    }
    if (any_result) {
      HIP_TRY(ctx, hipStreamSynchronize(st));
      for (int b = 0; b < B; ++b)
        if (n_pos[b] > 0) next_token[b] = ctx->out_host[b];
    }
  }
  for (int b = 0; b < B; ++b) kv->kv_len[b] = kv_len_now[b];
  return SPECASR_OK;
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
  const WsLayout L = ws_layout(ctx, batch);
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
  const WsLayout L = ws_layout(ctx, batch);
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
  const WsLayout L = ws_layout(ctx, B);
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
  const WsLayout L = ws_layout(ctx, B);
  const bool debug_timing = ctx->tune.debug;
  const auto t_begin = std::chrono::steady_clock::now();
  int32_t *o = reinterpret_cast<int32_t *>(ws + L.outs);
  const size_t BN = (size_t)B * c.max_nodes, MN = (size_t)c.max_nodes;
  int32_t *argmax_dev = o, *path_dev = o + BN, *len_dev = o + 2 * BN, *next_dev = len_dev + B;
  bool wide = false;
  std::vector<SeqGroup> groups = split_call(ctx, kv, tree, &wide);
  const WsLayout Lg = wide ? ws_layout_wide(ctx, B) : L;  // a wide call is one group in the wide buffers
  Lanes lanes{ctx, st, ws, L.total};
  s = lanes.begin(groups.size(), B);
  if (s != SPECASR_OK) return s;
  for (size_t gi = 0; gi < groups.size(); ++gi) {
    SeqGroup &grp = groups[gi];
    char *wl = wide ? ws + L.total * ws_lanes(ctx, B) : lanes.wsp(gi);
    hipStream_t sl = lanes.stream(gi);
    HostStep hs;
    build_step(ctx, &grp.tree, grp.kv.batch, grp.kv.kv_len, &hs);
    s = upload_meta(ctx, hs, wl, Lg, sl);
    if (s != SPECASR_OK) return s;
    ReadOut ro;
    ro.argmax = argmax_dev + grp.s0 * MN;
    ro.logits = out->logits ? out->logits + grp.s0 * MN * c.vocab : nullptr;
    s = forward_common(ctx, &grp.kv, &grp.tree, ro, wl, Lg, hs, sl, LayerSync(), wide);
    if (s != SPECASR_OK) return s;
    StepMeta m = device_meta(ctx, wl, Lg, grp.kv.batch, hs);
    KvGeom g{kv->capacity, c.n_layers, c.n_kv_heads, c.head_dim};
    launch_accept(m, c.max_nodes, argmax_dev + grp.s0 * MN, path_dev + grp.s0 * MN, len_dev + grp.s0, next_dev + grp.s0, sl);
    launch_compact(c.dtype, g, grp.kv.batch, c.max_nodes, m.kv_len, path_dev + grp.s0 * MN, len_dev + grp.s0, grp.kv.k, grp.kv.v, sl);
    HIP_TRY(ctx, hipGetLastError());
  }
  s = lanes.end();
  if (s != SPECASR_OK) return s;
  const size_t words = 2 * BN + 2 * (size_t)B;
  HIP_TRY(ctx, hipMemcpyAsync(ctx->out_host, o, words * 4, hipMemcpyDeviceToHost, st));
  const auto t_enqueued = std::chrono::steady_clock::now();
  HIP_TRY(ctx, hipStreamSynchronize(st));
  if (debug_timing) {  // host time spent enqueueing the step vs waiting for the GPU to finish it
    const auto t_done = std::chrono::steady_clock::now();
    fprintf(stderr, "[specasr] verify_tree: enqueue %.1f us, wait %.1f us\n",
            std::chrono::duration<double, std::micro>(t_enqueued - t_begin).count(),
            std::chrono::duration<double, std::micro>(t_done - t_enqueued).count());
  }
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

// ---- an entry point that allocates nothing ------------------------------------------------------
// specasr_accept_from_logits keeps the flattened tree metadata (per row: token, sequence, node,
// depth, parent, ancestor mask; per sequence: first row, node count) in the caller's workspace and
// fills it through pinned staging memory that the first call allocates.  The variant below keeps
// that block in a device array of the library instead and fills it with a kernel that receives one
// tree by value in its arguments, so nothing is allocated and nothing is copied.
}  // extern "C"

namespace {

constexpr int kStaticMaxBatch = SPECASR_STATIC_MAX_BATCH;
constexpr size_t kStaticScratchBytes =
    (meta_words(kStaticMaxBatch * SPECASR_MAX_NODES, kStaticMaxBatch) * 4 + 255) / 256 * 256;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

// Address of `scratch` on each device (every GPU holds its own copy of the array); looked up once
// per device, with that device current.
constexpr int kMaxDevices = 64;
std::mutex scratch_mu;
void *scratch_ptr[kMaxDevices] = {};

specasr_status static_scratch(specasr_ctx *ctx, char **out) {
  int dev = -1;
  HIP_TRY(ctx, hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return SPECASR_E_UNSUPPORTED;
  std::lock_guard<std::mutex> guard(scratch_mu);
  if (!scratch_ptr[dev]) {
    void *p = nullptr;
    HIP_TRY(ctx, hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p) return SPECASR_E_HIP;
    scratch_ptr[dev] = p;
  }
  *out = static_cast<char *>(scratch_ptr[dev]);
  return SPECASR_OK;
}

// One tree, passed by value in the kernel arguments.
struct TreeByValue {
  int32_t tokens[SPECASR_MAX_NODES];
  int32_t parents[SPECASR_MAX_NODES];
};

// Step 0 of the path on the device: rows row_start .. row_start + n - 1 of the metadata block (the
// layout build_step writes on the host, R = batch * max_nodes rows), lane = node.  The parent
// array was validated on the host (parents[i] < i), so the walk to the root ends within n steps.
__global__ __launch_bounds__(64) void tree_meta_kernel(TreeByValue t, int n, int seq, int row_start,
                                                       int R, int batch, int32_t *w) {
  const int i = threadIdx.x;
  if (i == 0) {
    w[10 * R + seq] = 0;                      // kv_len: acceptance has no cache position
    w[10 * R + batch + seq] = row_start;
    w[10 * R + 2 * batch + seq] = n;
  }
  if (i >= n) return;
  int depth = 0;
  uint64_t anc = 1ull << i;
  for (int p = t.parents[i], hops = 0; p >= 0 && hops < SPECASR_MAX_NODES; p = t.parents[p], ++hops) {
    anc |= 1ull << p;
    ++depth;
  }
  const int r = row_start + i;
  w[r] = t.tokens[i];
  w[R + r] = seq;
  w[2 * R + r] = i;
  w[3 * R + r] = depth;
  w[4 * R + r] = depth;                       // position and slot are zero-based here
  w[5 * R + r] = i;
  w[6 * R + r] = t.parents[i];
  w[7 * R + r] = 0;
  reinterpret_cast<uint64_t *>(w + 8 * R)[r] = anc;
}

}  // namespace

extern "C" {

specasr_status specasr_accept_from_logits_static(specasr_ctx *ctx, const specasr_tree *tree,
                                                 int32_t batch, const float *logits_dev,
                                                 int32_t *argmax_dev, int32_t *path_dev,
                                                 int32_t *accept_len_dev, int32_t *next_token_dev,
                                                 void *stream) {
  if (!ctx || !logits_dev || !argmax_dev || !path_dev || !accept_len_dev || !next_token_dev)
    return SPECASR_E_NULL;
  specasr_status s = validate_tree(ctx, tree, batch, nullptr, 0, false);
  if (s != SPECASR_OK) return s;
  if (batch > kStaticMaxBatch) return SPECASR_E_UNSUPPORTED;  // beyond what the device array holds
  char *sp = nullptr;
  s = static_scratch(ctx, &sp);
  if (s != SPECASR_OK) return s;
  hipStream_t st = (hipStream_t)stream;
  const specasr_config &c = ctx->cfg;
  const int R = batch * c.max_nodes;
  int32_t *w = reinterpret_cast<int32_t *>(sp);
  int rows = 0;
  for (int b = 0; b < batch; ++b) {
    const int n = tree->n_nodes[b];
    TreeByValue tv;
    memset(&tv, 0, sizeof tv);
    memcpy(tv.tokens, tree->tokens + (size_t)b * c.max_nodes, (size_t)n * 4);
    memcpy(tv.parents, tree->parents + (size_t)b * c.max_nodes, (size_t)n * 4);
    tree_meta_kernel<<<1, 64, 0, st>>>(tv, n, b, rows, R, batch, w);
    rows += n;
  }
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
  m.row_start = m.kv_len + batch;
  m.n_nodes = m.row_start + batch;
  m.rows = rows;
  m.batch = batch;
  m.kv_len0 = 0;
  m.n_nodes0 = tree->n_nodes[0];
  launch_argmax(m, logits_dev, true, c.max_nodes, c.vocab, argmax_dev, st);
  launch_accept(m, c.max_nodes, argmax_dev, path_dev, accept_len_dev, next_token_dev, st);
  HIP_TRY(ctx, hipGetLastError());
  return SPECASR_OK;
}

}  // extern "C"
