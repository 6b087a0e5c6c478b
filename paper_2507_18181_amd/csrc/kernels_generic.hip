// Dtype-generic stages of the tree-verification path: fp32 arithmetic on fp32 activations,
// weights and KV cache read in their storage type.  They serve fp32 models and are the
// fallback for shapes the MFMA kernels do not cover.  Also the integer stages (acceptance,
// KV compaction), which are shared by every path.
#include "kernels.h"

namespace specasr {

// --------------------------------------------------------------------------- rope table
// Sec. II-B: a tree node is verified as if decoded after its own branch, so its rotary
// position is kv_len + depth, shared by siblings.  Angles are formed in fp64 once per call.
__global__ void rope_table_kernel(const int32_t *pos, int rows, int half, int hd, double theta,
                                  float2 *cs) {
  int idx = blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= rows * half) return;
  int r = idx / half, j = idx - r * half;
  double ang = (double)pos[r] * pow(theta, -2.0 * (double)j / (double)hd);
  cs[idx] = make_float2((float)cos(ang), (float)sin(ang));
}

void launch_rope_table(const StepMeta &m, int hd, float theta, float2 *cs, hipStream_t st) {
  int half = hd / 2, n = m.rows * half;
  rope_table_kernel<<<(n + 255) / 256, 256, 0, st>>>(m.pos, m.rows, half, hd, (double)theta, cs);
}

// --------------------------------------------------------------------------- embedding gather
template <class T>
__global__ void embed_kernel(StepMeta m, const T *E, const T *in_emb, int max_nodes, int d, float *x) {
  int r = blockIdx.x;
  const T *src;
  if (in_emb != nullptr && m.use_embed[r])
    src = in_emb + ((int64_t)m.seq[r] * max_nodes + m.node[r]) * d;
  else
    src = E + (int64_t)m.token[r] * d;
  for (int c = threadIdx.x; c < d; c += blockDim.x) x[(int64_t)r * d + c] = to_f32(src[c]);
}

void launch_embed(const StepMeta &m, int dtype, const void *E, const void *in_emb, int max_nodes,
                  int d, float *x, hipStream_t st) {
  if (dtype == 1)
    embed_kernel<bf16_t><<<m.rows, 256, 0, st>>>(m, (const bf16_t *)E, (const bf16_t *)in_emb, max_nodes, d, x);
  else
    embed_kernel<float><<<m.rows, 256, 0, st>>>(m, (const float *)E, (const float *)in_emb, max_nodes, d, x);
}

// --------------------------------------------------------------------------- RMSNorm
template <class T>
__global__ void rmsnorm_kernel(const float *x, const T *g, int d, float eps, float *y) {
  __shared__ float red[16];
  const float *xr = x + (int64_t)blockIdx.x * d;
  float ss = 0.f;
  for (int c = threadIdx.x; c < d; c += blockDim.x) ss += xr[c] * xr[c];
  ss = block_sum(ss, red);
  float rs = 1.0f / sqrtf(ss / (float)d + eps);
  for (int c = threadIdx.x; c < d; c += blockDim.x)
    y[(int64_t)blockIdx.x * d + c] = xr[c] * rs * to_f32(g[c]);
}

void launch_rmsnorm(int dtype, const float *x, const void *g, int rows, int d, float eps, float *y,
                    hipStream_t st) {
  if (dtype == 1)
    rmsnorm_kernel<bf16_t><<<rows, 256, 0, st>>>(x, (const bf16_t *)g, d, eps, y);
  else
    rmsnorm_kernel<float><<<rows, 256, 0, st>>>(x, (const float *)g, d, eps, y);
}

// --------------------------------------------------------------------------- linear
// One wavefront owns OW output features and RB activation rows; lanes stride over k in
// 4-element vectors; a wave-wide sum finishes each dot product.  n_in % 4 == 0.
template <class T> struct Vec4;
template <> struct Vec4<float> {
  static __device__ __forceinline__ void load(const float *p, float w[4]) {
    float4 v = *reinterpret_cast<const float4 *>(p);
    w[0] = v.x; w[1] = v.y; w[2] = v.z; w[3] = v.w;
  }
};
template <> struct Vec4<bf16_t> {
  static __device__ __forceinline__ void load(const bf16_t *p, float w[4]) {
    uint2 v = *reinterpret_cast<const uint2 *>(p);
    w[0] = __uint_as_float(v.x << 16); w[1] = __uint_as_float(v.x & 0xffff0000u);
    w[2] = __uint_as_float(v.y << 16); w[3] = __uint_as_float(v.y & 0xffff0000u);
  }
};

template <class T, int RB, int OW>
__global__ __launch_bounds__(256) void linear_kernel(const T *W, int n_out, int n_in,
                                                     const float *a, int lda, float *y, int ldy,
                                                     int rows, int accumulate) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int o0 = (blockIdx.x * 4 + wave) * OW;
  const int r0 = blockIdx.y * RB;
  if (o0 >= n_out) return;
  float acc[OW][RB];
#pragma unroll
  for (int i = 0; i < OW; ++i)
#pragma unroll
    for (int j = 0; j < RB; ++j) acc[i][j] = 0.f;

  for (int k = lane * 4; k < n_in; k += 256) {
    float w[OW][4];
#pragma unroll
    for (int i = 0; i < OW; ++i) {
      int o = min(o0 + i, n_out - 1);
      Vec4<T>::load(W + (int64_t)o * n_in + k, w[i]);
    }
#pragma unroll
    for (int j = 0; j < RB; ++j) {
      int r = min(r0 + j, rows - 1);
      float4 av = *reinterpret_cast<const float4 *>(a + (int64_t)r * lda + k);
#pragma unroll
      for (int i = 0; i < OW; ++i)
        acc[i][j] += w[i][0] * av.x + w[i][1] * av.y + w[i][2] * av.z + w[i][3] * av.w;
    }
  }
#pragma unroll
  for (int i = 0; i < OW; ++i)
#pragma unroll
    for (int j = 0; j < RB; ++j) {
      float s = wave_sum(acc[i][j]);
      if (lane == 0 && o0 + i < n_out && r0 + j < rows) {
        float *dst = y + (int64_t)(r0 + j) * ldy + (o0 + i);
        *dst = accumulate ? (*dst + s) : s;
      }
    }
}

void launch_linear(int dtype, const void *W, int n_out, int n_in, const float *a, int lda,
                   float *y, int ldy, int rows, bool accumulate, hipStream_t st) {
  constexpr int RB = 8, OW = 2;
  dim3 grid((n_out + 4 * OW - 1) / (4 * OW), (rows + RB - 1) / RB);
  if (dtype == 1)
    linear_kernel<bf16_t, RB, OW><<<grid, 256, 0, st>>>((const bf16_t *)W, n_out, n_in, a, lda, y, ldy, rows, accumulate ? 1 : 0);
  else
    linear_kernel<float, RB, OW><<<grid, 256, 0, st>>>((const float *)W, n_out, n_in, a, lda, y, ldy, rows, accumulate ? 1 : 0);
}

// --------------------------------------------------------------------------- RoPE + KV append
// q: [rows][H*hd] rotated in place.  k, v: [rows][Hkv*hd]; k is rotated and both are written
// to cache slot kv_len + node of the row's sequence.
template <class T>
__global__ void rope_kv_kernel(StepMeta m, KvGeom g, int layer, int H, int Hkv, int hd,
                               const float2 *cs, float *q, const float *k, const float *v,
                               T *kc, T *vc) {
  const int r = blockIdx.x, half = hd / 2;
  const float2 *csr = cs + (int64_t)r * half;
  float *qr = q + (int64_t)r * H * hd;
  for (int idx = threadIdx.x; idx < H * half; idx += blockDim.x) {
    int a = idx / half, j = idx - a * half;
    float2 c = csr[j];
    float x0 = qr[a * hd + j], x1 = qr[a * hd + j + half];
    qr[a * hd + j] = x0 * c.x - x1 * c.y;
    qr[a * hd + j + half] = x1 * c.x + x0 * c.y;
  }
  const int seq = m.seq[r];
  const int64_t slot = m.slot[r];
  const float *kr = k + (int64_t)r * Hkv * hd, *vr = v + (int64_t)r * Hkv * hd;
  for (int idx = threadIdx.x; idx < Hkv * half; idx += blockDim.x) {
    int b = idx / half, j = idx - b * half;
    float2 c = csr[j];
    float x0 = kr[b * hd + j], x1 = kr[b * hd + j + half];
    int64_t base = g.row(seq, layer, b, slot);
    kc[base + j] = from_f32<T>(x0 * c.x - x1 * c.y);
    kc[base + j + half] = from_f32<T>(x1 * c.x + x0 * c.y);
    vc[base + j] = from_f32<T>(vr[b * hd + j]);
    vc[base + j + half] = from_f32<T>(vr[b * hd + j + half]);
  }
}

void launch_rope_kv(const StepMeta &m, const ModelDims &md, const KvGeom &g, int layer,
                    const float2 *cs, float *q, const float *k, const float *v, void *kc, void *vc,
                    hipStream_t st) {
  if (md.dtype == 1)
    rope_kv_kernel<bf16_t><<<m.rows, 256, 0, st>>>(m, g, layer, md.n_heads, md.n_kv_heads, md.head_dim, cs, q, k, v, (bf16_t *)kc, (bf16_t *)vc);
  else
    rope_kv_kernel<float><<<m.rows, 256, 0, st>>>(m, g, layer, md.n_heads, md.n_kv_heads, md.head_dim, cs, q, k, v, (float *)kc, (float *)vc);
}

// --------------------------------------------------------------------------- attention
// One block per (row, query head).  Keys are the cache slots [0, kv_len) plus the slots of
// the row's own root path (Sec. II-B: the 2D tree mask).  Online softmax over chunks of 256
// keys; scores, running maximum and sums in fp32.  hd <= 256 and 256 % hd == 0.
template <class T>
__global__ __launch_bounds__(256) void attention_generic_kernel(StepMeta m, KvGeom g, int layer,
                                                                int H, int Hkv, int hd,
                                                                const float *q, const T *kc,
                                                                const T *vc, float *out) {
  __shared__ float qs[256];
  __shared__ float sc[256];
  __shared__ float red[16];
  __shared__ float osum[256];
  const int r = blockIdx.x, a = blockIdx.y, tid = threadIdx.x;
  const int seq = m.seq[r], b = a / (H / Hkv);
  const int L = m.kv_len[seq], n = m.n_nodes[seq], T_all = L + n;
  const uint64_t anc = m.anc[r];
  const float scale = 1.0f / sqrtf((float)hd);
  if (tid < hd) qs[tid] = q[((int64_t)r * H + a) * hd + tid] * scale;
  __syncthreads();
  const T *kbase = kc + g.row(seq, layer, b, 0);
  const T *vbase = vc + g.row(seq, layer, b, 0);
  const int groups = 256 / hd, grp = tid / hd, c = tid - grp * hd;
  float m_run = -INFINITY, l_run = 0.f, o = 0.f;
  for (int t0 = 0; t0 < T_all; t0 += 256) {
    const int t = t0 + tid;
    const bool valid = t < T_all && (t < L || ((anc >> (t - L)) & 1ull));
    float s = -INFINITY;
    if (valid) {
      const T *kr = kbase + (int64_t)t * hd;
      float acc = 0.f;
      for (int e = 0; e < hd; ++e) acc += qs[e] * to_f32(kr[e]);
      s = acc;
    }
    const float cm = block_max(s, red);
    const float m_new = fmaxf(m_run, cm);
    if (m_new == -INFINITY) continue;  // a chunk with no visible key (uniform across the block)
    const float p = valid ? __expf(s - m_new) : 0.f;
    __syncthreads();
    sc[tid] = p;
    const float ls = block_sum(p, red);  // contains the barriers that publish sc[]
    const float alpha = (m_run == -INFINITY) ? 0.f : __expf(m_run - m_new);
    l_run = l_run * alpha + ls;
    o *= alpha;
    const int cnt = min(256, T_all - t0);
    for (int j = grp; j < cnt; j += groups) {
      float pj = sc[j];
      if (pj != 0.f) o += pj * to_f32(vbase[(int64_t)(t0 + j) * hd + c]);
    }
    m_run = m_new;
    __syncthreads();
  }
  osum[tid] = o;
  __syncthreads();
  if (tid < hd) {
    float tot = 0.f;
    for (int gi = 0; gi < groups; ++gi) tot += osum[gi * hd + tid];
    out[((int64_t)r * H + a) * hd + tid] = tot / l_run;
  }
}

void launch_attention_generic(const StepMeta &m, const ModelDims &md, const KvGeom &g, int layer,
                              const float *q, const void *kc, const void *vc, float *out,
                              hipStream_t st) {
  dim3 grid(m.rows, md.n_heads);
  if (md.dtype == 1)
    attention_generic_kernel<bf16_t><<<grid, 256, 0, st>>>(m, g, layer, md.n_heads, md.n_kv_heads, md.head_dim, q, (const bf16_t *)kc, (const bf16_t *)vc, out);
  else
    attention_generic_kernel<float><<<grid, 256, 0, st>>>(m, g, layer, md.n_heads, md.n_kv_heads, md.head_dim, q, (const float *)kc, (const float *)vc, out);
}

// --------------------------------------------------------------------------- SwiGLU
__global__ void swiglu_kernel(const float *gu, int rows, int F, float *t) {
  int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (int64_t)rows * F) return;
  int r = (int)(idx / F), f = (int)(idx - (int64_t)r * F);
  float gte = gu[(int64_t)r * 2 * F + f], up = gu[(int64_t)r * 2 * F + F + f];
  t[idx] = gte / (1.0f + __expf(-gte)) * up;
}

void launch_swiglu(const float *gu, int rows, int F, float *t, hipStream_t st) {
  int64_t n = (int64_t)rows * F;
  swiglu_kernel<<<(unsigned)((n + 255) / 256), 256, 0, st>>>(gu, rows, F, t);
}

// --------------------------------------------------------------------------- argmax
__global__ __launch_bounds__(256) void argmax_kernel(StepMeta m, const float *logits, int padded,
                                                     int max_nodes, int V, int32_t *argmax) {
  __shared__ float bv[4];
  __shared__ int bi[4];
  const int r = blockIdx.x;
  const int orow = m.seq[r] * max_nodes + m.node[r];
  const float *row = logits + (int64_t)(padded ? orow : r) * V;
  float best = -INFINITY;
  int besti = 0x7fffffff;
  for (int t = threadIdx.x; t < V; t += 256) {
    float v = row[t];
    if (v > best || (v == best && t < besti)) { best = v; besti = t; }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    float ov = __shfl_xor(best, o, 64);
    int oi = __shfl_xor(besti, o, 64);
    if (ov > best || (ov == best && oi < besti)) { best = ov; besti = oi; }
  }
  if ((threadIdx.x & 63) == 0) { bv[threadIdx.x >> 6] = best; bi[threadIdx.x >> 6] = besti; }
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int w = 1; w < 4; ++w)
      if (bv[w] > best || (bv[w] == best && bi[w] < besti)) { best = bv[w]; besti = bi[w]; }
    argmax[orow] = besti == 0x7fffffff ? 0 : besti;
  }
}

void launch_argmax(const StepMeta &m, const float *logits, bool padded_in, int max_nodes, int V,
                   int32_t *argmax, hipStream_t st) {
  argmax_kernel<<<m.rows, 256, 0, st>>>(m, logits, padded_in ? 1 : 0, max_nodes, V, argmax);
}

__global__ void scatter_logits_kernel(StepMeta m, const float *compact, int max_nodes, int V,
                                      float *padded) {
  const int r = blockIdx.x;
  const float *src = compact + (int64_t)r * V;
  float *dst = padded + (int64_t)(m.seq[r] * max_nodes + m.node[r]) * V;
  for (int t = blockIdx.y * blockDim.x + threadIdx.x; t < V; t += gridDim.y * blockDim.x) dst[t] = src[t];
}

void launch_scatter_logits(const StepMeta &m, const float *compact, int max_nodes, int V,
                           float *padded, hipStream_t st) {
  dim3 grid(m.rows, 8);
  scatter_logits_kernel<<<grid, 256, 0, st>>>(m, compact, max_nodes, V, padded);
}

// --------------------------------------------------------------------------- draft-side read-out
// Per row: the ids of the largest and the second largest logit and the softmax probability of
// the largest -- the draft model's normalised logit that is compared with a threshold, and the
// candidate of second highest probability that a sparse tree expands (Sec. IV-A, Sec. IV-C).
// Order: value descending, id ascending among equal values.
struct Top2 {
  float v1, v2;
  int i1, i2;
};
__device__ __forceinline__ bool top2_before(float a, int ia, float b, int ib) {
  return a > b || (a == b && ia < ib);
}
__device__ __forceinline__ void top2_push(Top2 &t, float v, int i) {
  if (top2_before(v, i, t.v1, t.i1)) {
    t.v2 = t.v1; t.i2 = t.i1; t.v1 = v; t.i1 = i;
  } else if (top2_before(v, i, t.v2, t.i2)) {
    t.v2 = v; t.i2 = i;
  }
}
__device__ __forceinline__ Top2 top2_merge(const Top2 &a, const Top2 &b) {
  Top2 r = a;
  top2_push(r, b.v1, b.i1);
  top2_push(r, b.v2, b.i2);
  return r;
}
__device__ __forceinline__ Top2 top2_wave(Top2 t) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    Top2 u;
    u.v1 = __shfl_xor(t.v1, o, 64); u.v2 = __shfl_xor(t.v2, o, 64);
    u.i1 = __shfl_xor(t.i1, o, 64); u.i2 = __shfl_xor(t.i2, o, 64);
    t = top2_merge(t, u);
  }
  return t;
}
constexpr int kNoId = 0x7fffffff;

// Stage 1, grid (blocks of 1024 ids, rows), block 256, 4 consecutive ids per thread.  SRC = 0: the
// logits are compact rows [rows][V]; SRC = 1: they are split-k partial sums (part_offset) that
// are summed here, multiplied by 1/rms of the row when nrm.ssq is set (second half of the final
// RMSNorm), and optionally stored into the caller's padded [batch][max_nodes][V] array.
// Record per (row, block): (v1, v2, sum of exp(v - v1) over the block), (i1, i2).
template <int SRC>
__global__ __launch_bounds__(256) void top2_blocks_kernel(StepMeta m, const float *src, int n_splits,
                                                          int ldp, RowNorm nrm, int V,
                                                          int max_nodes, float *logits_out,
                                                          float *rec_v, int *rec_i) {
  __shared__ Top2 wt[4];
  __shared__ float ws[4];
  const int r = blockIdx.y, rows = m.rows;
  const float rs = (SRC == 1 && nrm.ssq != nullptr) ? row_rms_scale(nrm, r) : 1.0f;
  const int v0 = (blockIdx.x * 256 + threadIdx.x) * 4;
  float vals[4] = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};
  if (v0 < V) {
    if (SRC == 0) {
#pragma unroll
      for (int i = 0; i < 4; ++i)
        if (v0 + i < V) vals[i] = src[(int64_t)r * V + v0 + i];
    } else {
      float4 a = make_float4(0.f, 0.f, 0.f, 0.f);
      for (int s = 0; s < n_splits; ++s) {
        const float4 p = *reinterpret_cast<const float4 *>(src + part_offset(s, r, v0, ldp >> 5, part_rows_pad(rows)));
        a.x += p.x; a.y += p.y; a.z += p.z; a.w += p.w;
      }
      const float t[4] = {a.x * rs, a.y * rs, a.z * rs, a.w * rs};
#pragma unroll
      for (int i = 0; i < 4; ++i)
        if (v0 + i < V) vals[i] = t[i];
    }
    if (logits_out) {
      float *dst = logits_out + ((int64_t)m.seq[r] * max_nodes + m.node[r]) * V + v0;
#pragma unroll
      for (int i = 0; i < 4; ++i)
        if (v0 + i < V) dst[i] = vals[i];
    }
  }
  Top2 t{-INFINITY, -INFINITY, kNoId, kNoId};
#pragma unroll
  for (int i = 0; i < 4; ++i)
    if (v0 + i < V) top2_push(t, vals[i], v0 + i);
  t = top2_wave(t);
  if ((threadIdx.x & 63) == 0) wt[threadIdx.x >> 6] = t;
  __syncthreads();
  t = top2_merge(top2_merge(wt[0], wt[1]), top2_merge(wt[2], wt[3]));
  float e = 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i)
    if (v0 + i < V) e += __expf(vals[i] - t.v1);
  e = wave_sum(e);
  if ((threadIdx.x & 63) == 0) ws[threadIdx.x >> 6] = e;
  __syncthreads();
  if (threadIdx.x == 0) {
    const int64_t o = (int64_t)r * gridDim.x + blockIdx.x;
    rec_v[o * 3] = t.v1;
    rec_v[o * 3 + 1] = t.v2;
    rec_v[o * 3 + 2] = (ws[0] + ws[1]) + (ws[2] + ws[3]);
    rec_i[o * 2] = t.i1;
    rec_i[o * 2 + 1] = t.i2;
  }
}

// Stage 2, one wavefront per row: merge the block records.  p1 = 1 / sum_b s_b * exp(v1_b - v1).
__global__ __launch_bounds__(64) void top2_merge_kernel(StepMeta m, const float *rec_v,
                                                        const int *rec_i, int n_blk, int max_nodes,
                                                        int32_t *top2, float *prob, int32_t *argmax) {
  const int r = blockIdx.x;
  Top2 t{-INFINITY, -INFINITY, kNoId, kNoId};
  for (int b = threadIdx.x; b < n_blk; b += 64) {
    const int64_t o = (int64_t)r * n_blk + b;
    const Top2 u{rec_v[o * 3], rec_v[o * 3 + 1], rec_i[o * 2], rec_i[o * 2 + 1]};
    t = top2_merge(t, u);
  }
  t = top2_wave(t);
  float sum = 0.f;
  for (int b = threadIdx.x; b < n_blk; b += 64) {
    const int64_t o = (int64_t)r * n_blk + b;
    sum += rec_v[o * 3 + 2] * __expf(rec_v[o * 3] - t.v1);
  }
  sum = wave_sum(sum);
  if (threadIdx.x == 0) {
    const int64_t orow = (int64_t)m.seq[r] * max_nodes + m.node[r];
    top2[orow * 2] = t.i1 == kNoId ? 0 : t.i1;
    top2[orow * 2 + 1] = t.i2 == kNoId ? -1 : t.i2;
    prob[orow] = 1.0f / sum;
    if (argmax) argmax[orow] = t.i1 == kNoId ? 0 : t.i1;
  }
}

int top2_blocks(int V) { return ((V + 3) / 4 + 255) / 256; }

void launch_top2(const StepMeta &m, const float *src, bool from_partials, int n_splits, int ldp,
                 const RowNorm &nrm, int V, int max_nodes, float *logits_out, float *rec_v, int *rec_i, int32_t *top2,
                 float *prob, int32_t *argmax, hipStream_t st) {
  const int n_blk = top2_blocks(V);
  dim3 grid(n_blk, m.rows);
  if (from_partials)
    top2_blocks_kernel<1><<<grid, 256, 0, st>>>(m, src, n_splits, ldp, nrm, V, max_nodes, logits_out, rec_v, rec_i);
  else
    top2_blocks_kernel<0><<<grid, 256, 0, st>>>(m, src, 0, 0, nrm, V, max_nodes, logits_out, rec_v, rec_i);
  top2_merge_kernel<<<m.rows, 64, 0, st>>>(m, rec_v, rec_i, n_blk, max_nodes, top2, prob, argmax);
}

// --------------------------------------------------------------------------- acceptance
// One wavefront per sequence, lane i = tree node i (trees have at most 64 nodes).
// Sec. II-B: draft tokens are accepted while they match the target's output and
// verification stops at the first failure.  A node matches when its token equals the
// target's greedy token at its parent; ballot gathers the match flags into one mask; a node is
// acceptable when its ancestor mask has no unmatched bit; the deepest acceptable node wins
// (lowest index among equals).
__global__ __launch_bounds__(64) void accept_kernel(StepMeta m, int max_nodes,
                                                    const int32_t *argmax, int32_t *path,
                                                    int32_t *accept_len, int32_t *next_token) {
  const int s = blockIdx.x, lane = threadIdx.x;
  const int n = m.n_nodes[s], r0 = m.row_start[s];
  const int32_t *am = argmax + (int64_t)s * max_nodes;
  bool matched = false;
  uint64_t anc = 0;
  int depth = 0;
  if (lane < n) {
    const int par = max(m.parent[r0 + lane], 0);
    matched = (lane == 0) || (m.token[r0 + lane] == am[par]);
    anc = m.anc[r0 + lane];
    depth = m.depth[r0 + lane];
  }
  const uint64_t mm = __ballot(matched);
  const bool ok = lane < n && (anc & ~mm) == 0ull;
  int key = ok ? (depth * 64 + (63 - lane)) : -1;
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) key = max(key, __shfl_xor(key, o, 64));
  const int win = 63 - (key & 63);
  const uint64_t wanc = __shfl(anc, win, 64);
  const int wdepth = key >> 6;
  int32_t *p = path + (int64_t)s * max_nodes;
  if (lane < max_nodes && lane > wdepth) p[lane] = -1;
  if (lane < n && ((wanc >> lane) & 1ull)) p[depth] = lane;
  if (lane == 0) {
    accept_len[s] = wdepth + 1;
    next_token[s] = am[win];
  }
}

void launch_accept(const StepMeta &m, int max_nodes, const int32_t *argmax, int32_t *path,
                   int32_t *accept_len, int32_t *next_token, hipStream_t st) {
  accept_kernel<<<m.batch, 64, 0, st>>>(m, max_nodes, argmax, path, accept_len, next_token);
}

// --------------------------------------------------------------------------- KV compaction
// Moves cache slot kv_len + path[k] to slot kv_len + k (k < accept_len) for one
// (sequence, layer, KV head, K|V) per block.  Since path is strictly increasing with
// path[k] >= k, a destination slot may be another move's source: every source row is read
// into registers, the block synchronises, and only then is anything written.
typedef __attribute__((ext_vector_type(4))) uint32_t mv16_t;  // one 16-byte unit of a cache row

template <int UNITS>
__global__ __launch_bounds__(256) void compact_kernel(KvGeom g, int max_nodes, int row_bytes,
                                                      const int32_t *kv_len, const int32_t *path,
                                                      const int32_t *accept_len, char *kc, char *vc,
                                                      int elem_bytes) {
  int idx = blockIdx.x;
  const int which = idx & 1; idx >>= 1;
  const int h = idx % g.n_kv_heads; idx /= g.n_kv_heads;
  const int layer = idx % g.n_layers;
  const int seq = idx / g.n_layers;
  const int len = accept_len[seq];
  const int32_t *p = path + (int64_t)seq * max_nodes;
  char *base = (which ? vc : kc) + g.row(seq, layer, h, kv_len[seq]) * elem_bytes;
  const int upr = row_bytes / 16;  // 16-byte units per row
  const int total = len * upr;
  if (total <= 256 * UNITS) {
    mv16_t regs[UNITS];
#pragma unroll
    for (int i = 0; i < UNITS; ++i) {
      int u = threadIdx.x + i * 256;
      if (u < total) {
        int k = u / upr, w = u - k * upr;
        int src = p[k];
        regs[i] = (mv16_t){0u, 0u, 0u, 0u};
        if (src != k) regs[i] = *reinterpret_cast<const mv16_t *>(base + (int64_t)src * row_bytes + w * 16);
      }
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < UNITS; ++i) {
      int u = threadIdx.x + i * 256;
      if (u < total) {
        int k = u / upr, w = u - k * upr;
        if (p[k] != k) *reinterpret_cast<mv16_t *>(base + (int64_t)k * row_bytes + w * 16) = regs[i];
      }
    }
  } else {
    // rows too large to stage at once: ascending order is safe because the source of move k'
    // (> k) lies beyond every destination written so far.
    for (int k = 0; k < len; ++k) {
      int src = p[k];
      if (src == k) continue;
      // one row is at most 1 KB = 64 units: every thread moves at most one
      mv16_t v = (mv16_t){0u, 0u, 0u, 0u};
      if ((int)threadIdx.x < upr)
        v = *reinterpret_cast<const mv16_t *>(base + (int64_t)src * row_bytes + threadIdx.x * 16);
      __syncthreads();
      if ((int)threadIdx.x < upr)
        *reinterpret_cast<mv16_t *>(base + (int64_t)k * row_bytes + threadIdx.x * 16) = v;
      __syncthreads();
    }
  }
}

void launch_compact(int dtype, const KvGeom &g, int batch, int max_nodes, const int32_t *kv_len,
                    const int32_t *path, const int32_t *accept_len, void *kc, void *vc,
                    hipStream_t st) {
  const int eb = dtype == 1 ? 2 : 4;
  const int row_bytes = g.head_dim * eb;  // multiple of 16: head_dim % 8 == 0
  const int blocks = batch * g.n_layers * g.n_kv_heads * 2;
  compact_kernel<8><<<blocks, 256, 0, st>>>(g, max_nodes, row_bytes, kv_len, path, accept_len,
                                           (char *)kc, (char *)vc, eb);
}

}  // namespace specasr
