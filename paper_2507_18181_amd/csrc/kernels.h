// Host-callable launchers of the device stages.  Every launcher only enqueues work on
// `st`; none synchronises or allocates.
#pragma once
#include "common.h"

namespace specasr {

struct ModelDims {
  int32_t n_layers, d_model, n_heads, n_kv_heads, head_dim, d_ffn, vocab;
  float rms_eps, rope_theta;
  int32_t dtype;  // 0 = fp32, 1 = bf16 storage
};

// ---- dtype-generic stages (fp32 arithmetic on fp32 activations) ----------
// rope table: cs[row][j] = (cos, sin)(pos[row] * theta^(-2j/hd)), computed in fp64
void launch_rope_table(const StepMeta &m, int hd, float theta, float2 *cs, hipStream_t st);
// x[row][:] = tok_embed[token[row]][:]  (or the caller's embedding row)
void launch_embed(const StepMeta &m, int dtype, const void *tok_embed, const void *input_embeds,
                  int max_nodes, int d, float *x, hipStream_t st);
// y[row][:] = x[row][:] * rsqrt(mean(x^2)+eps) * g
void launch_rmsnorm(int dtype, const float *x, const void *gain, int rows, int d, float eps,
                    float *y, hipStream_t st);
// y[row][o] (+)= sum_k W[o][k] * a[row][k]
void launch_linear(int dtype, const void *W, int n_out, int n_in, const float *a, int lda,
                   float *y, int ldy, int rows, bool accumulate, hipStream_t st);
// rotate q in place, rotate k, write k and v to their cache slots
void launch_rope_kv(const StepMeta &m, const ModelDims &md, const KvGeom &g, int layer,
                    const float2 *cs, float *q, const float *k, const float *v, void *kcache,
                    void *vcache, hipStream_t st);
// tree-masked attention of every (row, head) over cache slots [0, kv_len + n_nodes)
void launch_attention_generic(const StepMeta &m, const ModelDims &md, const KvGeom &g, int layer,
                              const float *q, const void *kcache, const void *vcache, float *out,
                              hipStream_t st);
// t = silu(gate) * up, gate/up interleaved as gu[row][0:F] and gu[row][F:2F]
void launch_swiglu(const float *gu, int rows, int F, float *t, hipStream_t st);
// argmax[seq][node] = lowest index of the maximum of the row's logits.  The logits are
// either compact ([rows][V], padded_in = false) or padded ([batch][max_nodes][V]).
void launch_argmax(const StepMeta &m, const float *logits, bool padded_in, int max_nodes, int V,
                   int32_t *argmax, hipStream_t st);
// copy compact logits rows into the caller's padded [batch][max_nodes][V] array
void launch_scatter_logits(const StepMeta &m, const float *compact, int max_nodes, int V,
                           float *padded, hipStream_t st);

// Draft-side read-out (Sec. IV-A, Sec. IV-C): top2[seq][node] = ids of the largest and second
// largest logit (value descending, id ascending; second = -1 if V == 1), prob[seq][node] = softmax
// probability of the first, argmax (optional) = the first id.  The logits are compact rows
// [rows][V], or (from_partials) split-k partial sums, times 1/rms of the row if nrm.ssq is set,
// that are also stored into logits_out ([batch][max_nodes][V], optional).  rec_v / rec_i: rows * top2_blocks(V) * 3 floats / 2 ints.
int top2_blocks(int V);
void launch_top2(const StepMeta &m, const float *src, bool from_partials, int n_splits, int ldp,
                 const RowNorm &nrm, int V, int max_nodes, float *logits_out, float *rec_v, int *rec_i, int32_t *top2,
                 float *prob, int32_t *argmax, hipStream_t st);

// ---- integer stages --------------------------------------------------------
// greedy acceptance, one wavefront per sequence; argmax in [batch][max_nodes] layout
void launch_accept(const StepMeta &m, int max_nodes, const int32_t *argmax, int32_t *path,
                   int32_t *accept_len, int32_t *next_token, hipStream_t st);
// in-place compaction of the accepted path's cache rows (path/accept_len on the device)
void launch_compact(int dtype, const KvGeom &g, int batch, int max_nodes, const int32_t *kv_len,
                    const int32_t *path, const int32_t *accept_len, void *kcache, void *vcache,
                    hipStream_t st);

}  // namespace specasr
