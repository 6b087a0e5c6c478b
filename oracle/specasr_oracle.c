/*
 * SpecASR tree-verification ORACLE  --  TEST INFRASTRUCTURE, NOT THE PRODUCT.
 *
 * A plain, slow, obviously-correct CPU implementation of what the verify step
 * of SpecASR computes: the target LLM decoder evaluates every token of a draft
 * token tree in one pass against a KV cache (paper Sec. II-B: tree-structured
 * speculative decoding with a 2D attention mask; Sec. IV-C: the sparse tree is
 * verified with that mask), and then accepts draft tokens that match the
 * target's own greedy output, stopping at the first failure (Sec. II-B,
 * "Draft-then-Verify").
 *
 * All floating-point arithmetic is IEEE double.  Weights and cache entries are
 * read in their storage type (fp32, bf16 bit patterns or fp64) and widened
 * exactly.  There is no blocking, fusion or reordering: each function takes the
 * steps in the order the definition states them.  OpenMP only distributes
 * independent output elements over host threads.
 *
 * Nothing here is shared with the HIP library.  Only tests, the smoke check and
 * the benchmark's cpu_baseline leg may call it.
 *
 * Decoder mathematics.  The paper names the decoder family only (Llama /
 * Vicuna / TinyLlama, Sec. II-A and Sec. V-A); the block used here is the
 * published Llama block: pre-norm RMSNorm, rotary position embedding with the
 * rotate-half pairing, (grouped-query) softmax attention, SwiGLU feed-forward,
 * no biases, untied LM head.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_F32 = 0, ORACLE_BF16 = 1, ORACLE_F64 = 2 };

typedef struct {
  int32_t n_layers, d_model, n_heads, n_kv_heads, head_dim, d_ffn, vocab;
  int32_t wdtype;  /* storage type of every weight tensor */
  double rms_eps, rope_theta;
} oracle_config;

typedef struct {
  const void *attn_norm, *wq, *wk, *wv, *wo, *ffn_norm, *w_gate, *w_up, *w_down;
} oracle_layer;

typedef struct {
  const void *tok_embed;  /* [vocab][d_model]  */
  const void *final_norm; /* [d_model]         */
  const void *lm_head;    /* [vocab][d_model]  */
  const oracle_layer *layers;
} oracle_weights;

/* ---- storage widening ---------------------------------------------------- */

/* Value a cache of storage type `dtype` holds after `v` is written to it: nearest fp32 for an
 * fp32 cache, nearest bf16 (ties to even, taken from that fp32) for a bf16 cache. */
static double store_round(double v, int dtype);

static double bf16_bits_to_double(uint16_t b) {
  uint32_t u = ((uint32_t)b) << 16;
  float f;
  memcpy(&f, &u, 4);
  return (double)f;
}

static void load_row(const void *base, int dtype, size_t off, size_t n, double *dst) {
  if (dtype == ORACLE_F32) {
    const float *p = (const float *)base + off;
    for (size_t i = 0; i < n; ++i) dst[i] = (double)p[i];
  } else if (dtype == ORACLE_BF16) {
    const uint16_t *p = (const uint16_t *)base + off;
    for (size_t i = 0; i < n; ++i) dst[i] = bf16_bits_to_double(p[i]);
  } else {
    const double *p = (const double *)base + off;
    for (size_t i = 0; i < n; ++i) dst[i] = p[i];
  }
}

/* ---- primitives (exported so the pins can test each one alone) ----------- */

/* RMSNorm: y_j = x_j / sqrt(mean_j(x_j^2) + eps) * g_j */
void oracle_rmsnorm(const double *x, const double *g, int n, double eps, double *y) {
  double ss = 0.0;
  for (int j = 0; j < n; ++j) ss += x[j] * x[j];
  double r = 1.0 / sqrt(ss / (double)n + eps);
  for (int j = 0; j < n; ++j) y[j] = x[j] * r * g[j];
}

/* Rotary embedding of one head vector at integer position pos.
 * Pair (j, j+hd/2) is rotated by the angle pos * theta^(-2j/hd). */
void oracle_rope(double *x, int hd, int64_t pos, double theta) {
  int half = hd / 2;
  for (int j = 0; j < half; ++j) {
    double ang = (double)pos * pow(theta, -2.0 * (double)j / (double)hd);
    double c = cos(ang), s = sin(ang);
    double a = x[j], b = x[j + half];
    x[j] = a * c - b * s;
    x[j + half] = b * c + a * s;
  }
}

/* Max-subtracted softmax in place. */
void oracle_softmax(double *s, int n) {
  double m = s[0];
  for (int j = 1; j < n; ++j)
    if (s[j] > m) m = s[j];
  double z = 0.0;
  for (int j = 0; j < n; ++j) {
    s[j] = exp(s[j] - m);
    z += s[j];
  }
  for (int j = 0; j < n; ++j) s[j] /= z;
}

double oracle_silu(double z) { return z / (1.0 + exp(-z)); }

/* y[i][o] = sum_k W[o][k] * a[i][k]   (W row-major [n_out][n_in], storage dtype) */
static void linear(const void *W, int dtype, int n_out, int n_in, const double *a, int n_rows,
                   double *y) {
#pragma omp parallel
  {
    double *wrow = (double *)malloc(sizeof(double) * (size_t)n_in);
#pragma omp for schedule(static)
    for (int o = 0; o < n_out; ++o) {
      load_row(W, dtype, (size_t)o * (size_t)n_in, (size_t)n_in, wrow);
      for (int i = 0; i < n_rows; ++i) {
        const double *ai = a + (size_t)i * (size_t)n_in;
        double acc = 0.0;
#pragma omp simd reduction(+ : acc)
        for (int k = 0; k < n_in; ++k) acc += wrow[k] * ai[k];
        y[(size_t)i * (size_t)n_out + (size_t)o] = acc;
      }
    }
    free(wrow);
  }
}

/* ---- step 0: tree preprocessing ------------------------------------------ */

/* depth[0]=0, depth[i]=depth[parent[i]]+1.  anc is an n*n 0/1 matrix with
 * anc[i*n+j]=1 iff j lies on the root-to-i path, i itself included: the 2D
 * tree mask (Sec. II-B), under which a node sees its own branch only.
 * Returns 0, or -1 when parents is not a rooted topological order. */
int oracle_tree_meta(const int32_t *parents, int n, int32_t *depth, uint8_t *anc) {
  if (n < 1 || parents[0] != -1) return -1;
  memset(anc, 0, (size_t)n * (size_t)n);
  depth[0] = 0;
  anc[0] = 1;
  for (int i = 1; i < n; ++i) {
    int p = parents[i];
    if (p < 0 || p >= i) return -1;
    depth[i] = depth[p] + 1;
    for (int j = 0; j < n; ++j) anc[(size_t)i * n + j] = anc[(size_t)p * n + j];
    anc[(size_t)i * n + i] = 1;
  }
  return 0;
}

static double store_round(double v, int dtype) {
  if (dtype == ORACLE_F64) return v;
  float f = (float)v;
  if (dtype == ORACLE_F32) return (double)f;
  uint32_t u;
  memcpy(&u, &f, 4);
  if ((u & 0x7f800000u) == 0x7f800000u) return (double)f; /* inf / nan unchanged */
  u += 0x7fffu + ((u >> 16) & 1u);
  return bf16_bits_to_double((uint16_t)(u >> 16));
}

/* ---- steps 1-8: decoder forward over the tree tokens ----------------------
 *
 * kcache/vcache : [n_layers][n_kv_heads][capacity][head_dim], storage cdtype;
 *                 only slots [0, L) are read; nothing is written.
 * tokens/parents: the tree, node 0 the root.
 * embeds        : optional [n][d_model] doubles; where use_embed[i] != 0 the
 *                 input row of node i is embeds[i] instead of the token
 *                 embedding (audio-embedding positions of a prefill chain).
 * Outputs (any may be NULL):
 *   logits [n][vocab], amax[n] (lowest index on exact ties),
 *   ktree/vtree [n_layers][n_kv_heads][n][head_dim]: the K (post-RoPE) and V
 *   rows computed for each node, indexed by node, as the cache holds them.
 * Node i is evaluated at position L + depth[i]; it attends to cache slots
 * [0, L) and to the tree nodes on its own root path.  The K/V rows of the tree
 * nodes are cache entries too (slot L + node): they take the cache's storage
 * type before attention reads them, like every other slot (no-op for an fp64
 * cache).
 */
int oracle_tree_forward(const oracle_config *cfg, const oracle_weights *w, const void *kcache,
                        const void *vcache, int cdtype, int64_t capacity, int64_t L,
                        const int32_t *tokens, const int32_t *parents, int n,
                        const double *embeds, const uint8_t *use_embed, double *logits,
                        int32_t *amax, double *ktree, double *vtree) {
  const int d = cfg->d_model, H = cfg->n_heads, Hkv = cfg->n_kv_heads, hd = cfg->head_dim;
  const int F = cfg->d_ffn, V = cfg->vocab, wt = cfg->wdtype;
  const int dq = H * hd, dkv = Hkv * hd, group = H / Hkv;
  if (n < 1 || L < 0 || L > capacity || H % Hkv != 0 || hd % 2 != 0) return -2;
  for (int i = 0; i < n; ++i) {
    int from_embed = embeds && use_embed && use_embed[i];
    if (!from_embed && (tokens[i] < 0 || tokens[i] >= V)) return -3;
  }

  int32_t *depth = (int32_t *)malloc(sizeof(int32_t) * n);
  uint8_t *anc = (uint8_t *)malloc((size_t)n * n);
  if (oracle_tree_meta(parents, n, depth, anc) != 0) {
    free(depth);
    free(anc);
    return -1;
  }

  double *x = (double *)malloc(sizeof(double) * (size_t)n * d);
  double *h = (double *)malloc(sizeof(double) * (size_t)n * d);
  double *q = (double *)malloc(sizeof(double) * (size_t)n * dq);
  double *k = (double *)malloc(sizeof(double) * (size_t)n * dkv);
  double *v = (double *)malloc(sizeof(double) * (size_t)n * dkv);
  double *att = (double *)malloc(sizeof(double) * (size_t)n * dq);
  double *proj = (double *)malloc(sizeof(double) * (size_t)n * d);
  double *gate = (double *)malloc(sizeof(double) * (size_t)n * F);
  double *up = (double *)malloc(sizeof(double) * (size_t)n * F);
  double *gain = (double *)malloc(sizeof(double) * (size_t)d);

  /* step 1: input rows */
  for (int i = 0; i < n; ++i) {
    if (embeds && use_embed && use_embed[i]) {
      memcpy(x + (size_t)i * d, embeds + (size_t)i * d, sizeof(double) * d);
    } else {
      load_row(w->tok_embed, wt, (size_t)tokens[i] * d, d, x + (size_t)i * d);
    }
  }

  for (int l = 0; l < cfg->n_layers; ++l) {
    const oracle_layer *lw = &w->layers[l];

    /* step 2: pre-attention norm and Q, K, V projections */
    load_row(lw->attn_norm, wt, 0, d, gain);
    for (int i = 0; i < n; ++i)
      oracle_rmsnorm(x + (size_t)i * d, gain, d, cfg->rms_eps, h + (size_t)i * d);
    linear(lw->wq, wt, dq, d, h, n, q);
    linear(lw->wk, wt, dkv, d, h, n, k);
    linear(lw->wv, wt, dkv, d, h, n, v);

    /* step 3: rotary embedding keyed by depth, not by slot */
    for (int i = 0; i < n; ++i) {
      int64_t pos = L + depth[i];
      for (int a = 0; a < H; ++a) oracle_rope(q + (size_t)i * dq + (size_t)a * hd, hd, pos, cfg->rope_theta);
      for (int b = 0; b < Hkv; ++b) oracle_rope(k + (size_t)i * dkv + (size_t)b * hd, hd, pos, cfg->rope_theta);
    }
    /* the rows are appended to the cache: they take its storage type */
    for (size_t e = 0; e < (size_t)n * dkv; ++e) {
      k[e] = store_round(k[e], cdtype);
      v[e] = store_round(v[e], cdtype);
    }
    if (ktree && vtree) {
      for (int b = 0; b < Hkv; ++b)
        for (int i = 0; i < n; ++i) {
          size_t dst = (((size_t)l * Hkv + b) * n + i) * hd;
          memcpy(ktree + dst, k + (size_t)i * dkv + (size_t)b * hd, sizeof(double) * hd);
          memcpy(vtree + dst, v + (size_t)i * dkv + (size_t)b * hd, sizeof(double) * hd);
        }
    }

    /* step 4: attention over the cached prefix and the node's own ancestors */
#pragma omp parallel
    {
      double *sc = (double *)malloc(sizeof(double) * (size_t)(L + n));
      double *krow = (double *)malloc(sizeof(double) * hd);
      int32_t *src = (int32_t *)malloc(sizeof(int32_t) * (size_t)(L + n));
#pragma omp for collapse(2) schedule(static)
      for (int i = 0; i < n; ++i) {
        for (int a = 0; a < H; ++a) {
          const int b = a / group;
          const double *qi = q + (size_t)i * dq + (size_t)a * hd;
          const size_t cbase = ((size_t)l * Hkv + b) * (size_t)capacity * hd;
          const double scale = 1.0 / sqrt((double)hd);
          int m = 0;
          for (int64_t s = 0; s < L; ++s) {
            load_row(kcache, cdtype, cbase + (size_t)s * hd, hd, krow);
            double acc = 0.0;
            for (int c = 0; c < hd; ++c) acc += qi[c] * krow[c];
            sc[m] = acc * scale;
            src[m++] = (int32_t)s;
          }
          for (int j = 0; j < n; ++j) {
            if (!anc[(size_t)i * n + j]) continue;
            const double *kj = k + (size_t)j * dkv + (size_t)b * hd;
            double acc = 0.0;
            for (int c = 0; c < hd; ++c) acc += qi[c] * kj[c];
            sc[m] = acc * scale;
            src[m++] = -(j + 1); /* tree node j */
          }
          oracle_softmax(sc, m);
          double *o = att + (size_t)i * dq + (size_t)a * hd;
          for (int c = 0; c < hd; ++c) o[c] = 0.0;
          for (int t = 0; t < m; ++t) {
            if (src[t] >= 0) {
              load_row(vcache, cdtype, cbase + (size_t)src[t] * hd, hd, krow);
              for (int c = 0; c < hd; ++c) o[c] += sc[t] * krow[c];
            } else {
              const double *vj = v + (size_t)(-src[t] - 1) * dkv + (size_t)b * hd;
              for (int c = 0; c < hd; ++c) o[c] += sc[t] * vj[c];
            }
          }
        }
      }
      free(sc);
      free(krow);
      free(src);
    }

    /* step 5: output projection, residual */
    linear(lw->wo, wt, d, dq, att, n, proj);
    for (size_t e = 0; e < (size_t)n * d; ++e) x[e] += proj[e];

    /* step 6: pre-FFN norm, gate and up projections, SwiGLU */
    load_row(lw->ffn_norm, wt, 0, d, gain);
    for (int i = 0; i < n; ++i)
      oracle_rmsnorm(x + (size_t)i * d, gain, d, cfg->rms_eps, h + (size_t)i * d);
    linear(lw->w_gate, wt, F, d, h, n, gate);
    linear(lw->w_up, wt, F, d, h, n, up);
    for (size_t e = 0; e < (size_t)n * F; ++e) gate[e] = oracle_silu(gate[e]) * up[e];

    /* step 7: down projection, residual */
    linear(lw->w_down, wt, d, F, gate, n, proj);
    for (size_t e = 0; e < (size_t)n * d; ++e) x[e] += proj[e];
  }

  /* step 8: final norm, LM head, per-node argmax */
  if (logits || amax) {
    double *lg = logits ? logits : (double *)malloc(sizeof(double) * (size_t)n * V);
    load_row(w->final_norm, wt, 0, d, gain);
    for (int i = 0; i < n; ++i)
      oracle_rmsnorm(x + (size_t)i * d, gain, d, cfg->rms_eps, h + (size_t)i * d);
    linear(w->lm_head, wt, V, d, h, n, lg);
    if (amax) {
      for (int i = 0; i < n; ++i) {
        const double *row = lg + (size_t)i * V;
        int best = 0;
        for (int t = 1; t < V; ++t)
          if (row[t] > row[best]) best = t;
        amax[i] = best;
      }
    }
    if (!logits) free(lg);
  }

  free(depth); free(anc); free(x); free(h); free(q); free(k); free(v);
  free(att); free(proj); free(gate); free(up); free(gain);
  return 0;
}

/* ---- step 9: greedy acceptance --------------------------------------------
 *
 * The root (node 0) is the last committed token and is always accepted.  A
 * draft node i>0 is "matched" when its token equals the target's greedy output
 * at its parent.  A node is acceptable when every node on its root path is
 * matched (verification stops at the first failing token, Sec. II-B).  The
 * result is the deepest acceptable node, lowest index among equals; path is
 * the root-to-result node list; next_token is the target's output there (the
 * token the target itself would emit after the accepted ones).
 */
int oracle_accept(const int32_t *tokens, const int32_t *parents, const int32_t *amax, int n,
                  int32_t *path, int32_t *accept_len, int32_t *next_token) {
  int32_t *depth = (int32_t *)malloc(sizeof(int32_t) * n);
  uint8_t *anc = (uint8_t *)malloc((size_t)n * n);
  if (oracle_tree_meta(parents, n, depth, anc) != 0) {
    free(depth);
    free(anc);
    return -1;
  }
  int best = 0;
  for (int i = 0; i < n; ++i) {
    int ok = 1;
    for (int j = 1; j < n; ++j)
      if (anc[(size_t)i * n + j] && tokens[j] != amax[parents[j]]) ok = 0;
    if (ok && depth[i] > depth[best]) best = i;
  }
  int len = depth[best] + 1;
  for (int node = best, kk = len - 1; kk >= 0; --kk, node = parents[node]) path[kk] = node;
  *accept_len = len;
  *next_token = amax[best];
  free(depth);
  free(anc);
  return 0;
}

/*
 * Draft-side read-out of logit rows.  The draft model's confidence in a predicted token is its
 * normalised logit, i.e. its softmax probability, which is compared with a threshold to decide
 * where a draft is cut or marked as uncertain (Sec. IV-A; 0.4 in Sec. V-A); at uncertain positions
 * the tokens of highest probability are kept and the one of second highest probability is the
 * one expanded into a branch (Sec. IV-C, Sec. V-C).
 *
 * For each of the n rows x[0..V):
 *   top[2r]   = the id of the largest logit (lowest id among equals)
 *   top[2r+1] = the id of the largest logit among the other ids (lowest id among equals),
 *               -1 when V == 1
 *   p1[r]     = exp(x[top0]) / sum_j exp(x[j]), evaluated as 1 / sum_j exp(x[j] - x[top0])
 */
int oracle_top2(const double *logits, int n, int V, int32_t *top, double *p1) {
  if (n < 0 || V < 1) return -1;
  for (int r = 0; r < n; ++r) {
    const double *x = logits + (size_t)r * V;
    int a = 0;
    for (int j = 1; j < V; ++j)
      if (x[j] > x[a]) a = j;
    int b = -1;
    for (int j = 0; j < V; ++j) {
      if (j == a) continue;
      if (b < 0 || x[j] > x[b]) b = j;
    }
    double sum = 0.0;
    for (int j = 0; j < V; ++j) sum += exp(x[j] - x[a]);
    top[2 * r] = a;
    top[2 * r + 1] = b;
    p1[r] = 1.0 / sum;
  }
  return 0;
}

int oracle_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}
