// bf16 MFMA stages of the tree-verification path for gfx950 (CDNA4, wave64).
//
// The projections of the decoder are skinny GEMMs: at most 64 tree-node rows against every
// weight of the model, so each weight byte is used once per call and the stage is bound by HBM
// bandwidth.  Design:
//   * Weights are repacked once (specasr_create) into MFMA-operand order: the matrix is cut into
//     tiles of 32 output features x 16 input features; one tile is 1 KB laid out exactly as the A
//     operand of v_mfma_f32_32x32x16_bf16 (lane l holds row l%32, k = 8*(l/32)..+7), and the tiles
//     of one 32-row band are contiguous along k.  A wavefront therefore streams its band with
//     one fully coalesced 16-byte load per lane per tile and feeds it to the matrix core with no
//     shuffle and no LDS round trip.
//   * The activations (the B operand, <= 64 rows) are tiny: the workgroup stages its k-chunk of
//     them into LDS once, already in B-operand order, and every wavefront re-reads them from there.
//     They are carried as TWO bf16 planes, hi = bf16(v) and lo = bf16(v - hi), and every weight
//     tile is multiplied with both: the products are exact in fp32, so the projections see the
//     activations to 16 mantissa bits.  The matrix cores have >10x headroom on this stage; the
//     extra MFMA is what keeps 22-32 layers inside the 2e-2 logit tolerance.
//   * Work is split over (k-chunk, band group) so that a few thousand wavefronts each stream a
//     contiguous span with a ring of loads in flight; partial sums over the k-chunks are written
//     to a small fp32 buffer and reduced, in a fixed order, by the consumer stage.
#include "kernels.h"
#include "kernels_mfma.h"

namespace specasr {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

__device__ __forceinline__ u32x4 load_stream(const u32x4 *p) { return __builtin_nontemporal_load(p); }

// --------------------------------------------------------------------------- weight repack
// dst tile (band, kt), lane l, element i  <-  src[band*32 + l%32][kt*16 + 8*(l/32) + i]
// Rows >= n_out (padding of the last band) and columns >= K (padding of k to a whole number of
// kGemmU-tile batches) are zero.  `band0` is the first packed band written, so several source
// matrices can be concatenated band-aligned into one packed matrix.
__global__ void repack_kernel(const uint16_t *src, int n_out, int K, int ksteps_pad, uint16_t *dst,
                              int band0) {
  const int64_t tile = blockIdx.x;  // over bands * ksteps_pad
  const int band = (int)(tile / ksteps_pad), kt = (int)(tile - (int64_t)band * ksteps_pad);
  const int l = threadIdx.x;  // 64 lanes
  const int row = band * 32 + (l & 31);
  const int col = kt * 16 + 8 * (l >> 5);
  u32x4 v = (u32x4){0u, 0u, 0u, 0u};
  if (row < n_out && col < K) v = *reinterpret_cast<const u32x4 *>(src + (int64_t)row * K + col);
  reinterpret_cast<u32x4 *>(dst)[((int64_t)(band0 + band) * ksteps_pad + kt) * 64 + l] = v;
}

void launch_repack(const void *src, int n_out, int K, int ksteps_pad, void *dst, int band0,
                   hipStream_t st) {
  const int bands = (n_out + 31) / 32;
  const int64_t tiles = (int64_t)bands * ksteps_pad;
  repack_kernel<<<(unsigned)tiles, 64, 0, st>>>((const uint16_t *)src, n_out, K, ksteps_pad, (uint16_t *)dst, band0);
}

// --------------------------------------------------------------------------- skinny GEMM
// part[s][row][o] = sum over k in chunk s of X[row][k] * W[o][k]
// grid.x = n_splits * n_groups; block = 256 (4 wavefronts); wavefront w of group g owns bands
// [(g*4+w)*bpw, +bpw).  LDS: X chunk in B-operand order, [kstep][NB][hi|lo][64 lanes] x 16 bytes.
// Every chunk holds a whole number of U-tile batches (the packed k extent is padded to that), so
// the steady-state loop is branch-free: U unconditional loads stay in flight per lane, the ring
// runs on across band boundaries, and at the very end it re-reads the last batch (unused).
template <int NB, int U>
__global__ __launch_bounds__(256) void gemm_skinny_kernel(const u32x4 *__restrict__ Wp,
                                                          const uint16_t *__restrict__ X,
                                                          const uint16_t *__restrict__ Xlo, int ldx,
                                                          int K, float *__restrict__ part, int ldo,
                                                          int rows, int n_bands, int ksteps_all,
                                                          int n_splits, int chunk_steps, int bpw) {
  extern __shared__ u32x4 lds[];
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const int s = blockIdx.x % n_splits, grp = blockIdx.x / n_splits;
  const int ks0 = s * chunk_steps;
  const int nks = min(chunk_steps, ksteps_all - ks0);  // k-steps of this chunk, a multiple of U
  const int b0 = min((grp * 4 + wave) * bpw, n_bands), b1 = min(b0 + bpw, n_bands);
  const u32x4 *wbase = Wp + (int64_t)ks0 * 64 + lane;
  const int64_t band_stride = (int64_t)ksteps_all * 64;

  // start the weight stream before anything else
  u32x4 buf[U];
  {
    const u32x4 *p = wbase + (int64_t)min(b0, n_bands - 1) * band_stride;
#pragma unroll
    for (int u = 0; u < U; ++u) buf[u] = load_stream(p + 64 * u);
  }
  // stage the activation chunk: slot (kstep, nb, l) <- X[nb*32 + l%32][16*(ks0+kstep) + 8*(l/32) ..+7]
  for (int idx = threadIdx.x; idx < nks * NB * 128; idx += 256) {
    const int l = idx & 63, blk = idx >> 6;
    const int part_lo = blk & 1, nb = (blk >> 1) % NB, kstep = (blk >> 1) / NB;
    const int r = nb * 32 + (l & 31);
    const int col = 16 * (ks0 + kstep) + 8 * (l >> 5);
    u32x4 v = (u32x4){0u, 0u, 0u, 0u};
    if (r < rows && col < K) v = *reinterpret_cast<const u32x4 *>((part_lo ? Xlo : X) + (int64_t)r * ldx + col);
    lds[idx] = v;
  }
  __syncthreads();

  for (int band = b0; band < b1; ++band) {
    // two accumulator sets per node group (hi and lo plane): independent MFMA chains
    f32x16 acc[NB][2];
#pragma unroll
    for (int n = 0; n < NB; ++n)
#pragma unroll
      for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int j = 0; j < 16; ++j) acc[n][h][j] = 0.f;
    for (int kb = 0; kb < nks; kb += U) {
      // where the next batch of this wavefront's stream lives
      int nband = band, nk = kb + U;
      if (nk >= nks) { nk = 0; ++nband; }
      if (nband >= b1) { nband = band; nk = kb; }
      const u32x4 *pn = wbase + (int64_t)nband * band_stride + (int64_t)nk * 64;
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const bf16x8 a = __builtin_bit_cast(bf16x8, buf[u]);
#pragma unroll
        for (int n = 0; n < NB; ++n) {
          const bf16x8 bh = __builtin_bit_cast(bf16x8, lds[(((kb + u) * NB + n) * 2) * 64 + lane]);
          const bf16x8 bl = __builtin_bit_cast(bf16x8, lds[(((kb + u) * NB + n) * 2 + 1) * 64 + lane]);
          acc[n][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, bh, acc[n][0], 0, 0, 0);
          acc[n][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, bl, acc[n][1], 0, 0, 0);
        }
        buf[u] = load_stream(pn + 64 * u);  // refill the slot just consumed
      }
    }
    // C layout: lane l holds node column l%32 and output rows 8*(j/4) + 4*(l/32) + j%4
#pragma unroll
    for (int n = 0; n < NB; ++n) {
      const int r = n * 32 + (lane & 31);
      if (r < rows) {
        float *dst = part + ((int64_t)s * rows + r) * ldo + band * 32 + 4 * (lane >> 5);
#pragma unroll
        for (int q = 0; q < 4; ++q)
          *reinterpret_cast<float4 *>(dst + 8 * q) =
              make_float4(acc[n][0][4 * q] + acc[n][1][4 * q], acc[n][0][4 * q + 1] + acc[n][1][4 * q + 1],
                          acc[n][0][4 * q + 2] + acc[n][1][4 * q + 2], acc[n][0][4 * q + 3] + acc[n][1][4 * q + 3]);
      }
    }
  }
}

void launch_gemm_skinny(const PackedMatrix &W, const uint16_t *X, const uint16_t *Xlo, int ldx,
                        int rows, float *part, const GemmPlan &plan, hipStream_t st) {
  const int groups = (W.n_bands + 4 * plan.bands_per_wave - 1) / (4 * plan.bands_per_wave);
  const dim3 grid(groups * plan.n_splits);
  const int nb = rows <= 32 ? 1 : 2;
  const size_t lds = (size_t)plan.chunk_steps * nb * 2 * 64 * 16;
  if (nb == 1)
    gemm_skinny_kernel<1, kGemmU><<<grid, 256, lds, st>>>((const u32x4 *)W.data, X, Xlo, ldx, W.k_real, part, W.ldo, rows, W.n_bands, W.ksteps, plan.n_splits, plan.chunk_steps, plan.bands_per_wave);
  else
    gemm_skinny_kernel<2, kGemmU><<<grid, 256, lds, st>>>((const u32x4 *)W.data, X, Xlo, ldx, W.k_real, part, W.ldo, rows, W.n_bands, W.ksteps, plan.n_splits, plan.chunk_steps, plan.bands_per_wave);
}

hipError_t gemm_skinny_set_lds_limit() {
  hipError_t e = hipFuncSetAttribute((const void *)gemm_skinny_kernel<1, kGemmU>, hipFuncAttributeMaxDynamicSharedMemorySize, kGemmMaxLds);
  if (e != hipSuccess) return e;
  return hipFuncSetAttribute((const void *)gemm_skinny_kernel<2, kGemmU>, hipFuncAttributeMaxDynamicSharedMemorySize, kGemmMaxLds);
}

// --------------------------------------------------------------------------- consumers of partial sums
// x[r][:] += sum_s part[s][r][:]   (n_splits may be 0: plain norm)
// hb[r][:]  = bf16( x[r][:] * rsqrt(mean(x^2) + eps) * gain )
__global__ __launch_bounds__(1024) void residual_norm_kernel(float *x, const float *part, int n_splits,
                                                             int rows, int ldp, const uint16_t *gain,
                                                             int d, float eps, uint16_t *hb,
                                                             uint16_t *hb_lo) {
  __shared__ float red[16];
  const int r = blockIdx.x;
  float *xr = x + (int64_t)r * d;
  float ss = 0.f;
  for (int c = threadIdx.x * 4; c < d; c += 4096) {
    float4 v = *reinterpret_cast<const float4 *>(xr + c);
    const float *pp = part + (int64_t)r * ldp + c;
    const int64_t sstride = (int64_t)rows * ldp;
    int s = 0;
    for (; s + 4 <= n_splits; s += 4) {  // four independent loads in flight, summed in split order
      const float4 p0 = *reinterpret_cast<const float4 *>(pp + (s + 0) * sstride);
      const float4 p1 = *reinterpret_cast<const float4 *>(pp + (s + 1) * sstride);
      const float4 p2 = *reinterpret_cast<const float4 *>(pp + (s + 2) * sstride);
      const float4 p3 = *reinterpret_cast<const float4 *>(pp + (s + 3) * sstride);
      v.x += p0.x; v.y += p0.y; v.z += p0.z; v.w += p0.w;
      v.x += p1.x; v.y += p1.y; v.z += p1.z; v.w += p1.w;
      v.x += p2.x; v.y += p2.y; v.z += p2.z; v.w += p2.w;
      v.x += p3.x; v.y += p3.y; v.z += p3.z; v.w += p3.w;
    }
    for (; s < n_splits; ++s) {
      const float4 p = *reinterpret_cast<const float4 *>(pp + s * sstride);
      v.x += p.x; v.y += p.y; v.z += p.z; v.w += p.w;
    }
    if (n_splits > 0) *reinterpret_cast<float4 *>(xr + c) = v;
    ss += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
  }
  ss = block_sum(ss, red);
  const float rs = 1.0f / sqrtf(ss / (float)d + eps);
  for (int c = threadIdx.x * 4; c < d; c += 4096) {
    const float4 v = *reinterpret_cast<const float4 *>(xr + c);
    const uint2 g = *reinterpret_cast<const uint2 *>(gain + c);
    const float y[4] = {v.x * rs * bf16_bits_to_f32(g.x & 0xffffu), v.y * rs * bf16_bits_to_f32(g.x >> 16),
                        v.z * rs * bf16_bits_to_f32(g.y & 0xffffu), v.w * rs * bf16_bits_to_f32(g.y >> 16)};
    uint16_t hi[4], lo[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) split_bf16(y[i], hi[i], lo[i]);
    *reinterpret_cast<uint2 *>(hb + (int64_t)r * d + c) =
        make_uint2((uint32_t)hi[0] | ((uint32_t)hi[1] << 16), (uint32_t)hi[2] | ((uint32_t)hi[3] << 16));
    *reinterpret_cast<uint2 *>(hb_lo + (int64_t)r * d + c) =
        make_uint2((uint32_t)lo[0] | ((uint32_t)lo[1] << 16), (uint32_t)lo[2] | ((uint32_t)lo[3] << 16));
  }
}

void launch_residual_norm(float *x, const float *part, int n_splits, int rows, int ldp,
                          const void *gain, int d, float eps, uint16_t *hb, uint16_t *hb_lo,
                          hipStream_t st) {
  residual_norm_kernel<<<rows, 1024, 0, st>>>(x, part, n_splits, rows, ldp, (const uint16_t *)gain, d, eps, hb, hb_lo);
}

// q, k, v = sum of partials; rotary embedding at the node's depth position (Sec. II-B: each
// branch is verified as its own sequence, so position = kv_len + depth).  Outputs: q either as
// fp32 [rows][H*hd] (generic attention) or as bf16 pre-multiplied by 1/sqrt(hd) (MFMA
// attention); k, v -> bf16 cache slot kv_len + node.  Packed columns: [q | pad | k | pad | v].
__global__ __launch_bounds__(256) void qkv_finish_kernel(StepMeta m, KvGeom g, int layer, int H, int Hkv,
                                                         int hd, const float *part, int n_splits,
                                                         int ldp, int col_k, int col_v,
                                                         const float2 *cs, float *q, uint16_t *qb,
                                                         uint16_t *qb_lo, float qscale, uint16_t *kc,
                                                         uint16_t *vc) {
  const int r = blockIdx.y, half = hd / 2, rows = m.rows;
  const int idx = blockIdx.x * 256 + threadIdx.x;
  if (idx >= (H + Hkv) * half) return;
  const int a = idx / half, j = idx - a * half;
  const float2 c = cs[(int64_t)r * half + j];
  const float *pr = part + (int64_t)r * ldp;
  const int64_t sstride = (int64_t)rows * ldp;
  auto val = [&](int col) {
    float v = 0.f;
    for (int s = 0; s < n_splits; ++s) v += pr[s * sstride + col];
    return v;
  };
  if (a < H) {
    const float x0 = val(a * hd + j), x1 = val(a * hd + j + half);
    const float y0 = x0 * c.x - x1 * c.y, y1 = x1 * c.x + x0 * c.y;
    const int64_t o = ((int64_t)r * H + a) * hd + j;
    if (qb) {
      split_bf16(y0 * qscale, qb[o], qb_lo[o]);
      split_bf16(y1 * qscale, qb[o + half], qb_lo[o + half]);
    } else {
      q[o] = y0;
      q[o + half] = y1;
    }
  } else {
    const int b = a - H;
    const float x0 = val(col_k + b * hd + j), x1 = val(col_k + b * hd + j + half);
    const int64_t base = g.row(m.seq[r], layer, b, m.slot[r]);
    kc[base + j] = f32_to_bf16_bits(x0 * c.x - x1 * c.y);
    kc[base + j + half] = f32_to_bf16_bits(x1 * c.x + x0 * c.y);
    vc[base + j] = f32_to_bf16_bits(val(col_v + b * hd + j));
    vc[base + j + half] = f32_to_bf16_bits(val(col_v + b * hd + j + half));
  }
}

void launch_qkv_finish(const StepMeta &m, const ModelDims &md, const KvGeom &g, int layer,
                       const float *part, int n_splits, int ldp, int col_k, int col_v,
                       const float2 *cs, float *q, uint16_t *qb, uint16_t *qb_lo, void *kc, void *vc,
                       hipStream_t st) {
  const int items = (md.n_heads + md.n_kv_heads) * (md.head_dim / 2);
  dim3 grid((items + 255) / 256, m.rows);
  qkv_finish_kernel<<<grid, 256, 0, st>>>(m, g, layer, md.n_heads, md.n_kv_heads, md.head_dim, part, n_splits, ldp, col_k, col_v, cs, q, qb, qb_lo, 1.0f / sqrtf((float)md.head_dim), (uint16_t *)kc, (uint16_t *)vc);
}

// t[r][f] = bf16( silu(sum_s gate) * (sum_s up) ); gate at column f, up at column col_up + f
__global__ __launch_bounds__(256) void swiglu_finish_kernel(const float *part, int n_splits, int rows,
                                                            int ldp, int col_up, int F, uint16_t *t,
                                                            uint16_t *t_lo) {
  const int r = blockIdx.y;
  const int f = (blockIdx.x * 256 + threadIdx.x) * 4;
  if (f >= F) return;
  float4 gt = make_float4(0.f, 0.f, 0.f, 0.f), up = gt;
  for (int s = 0; s < n_splits; ++s) {
    const float *p = part + ((int64_t)s * rows + r) * ldp;
    const float4 a = *reinterpret_cast<const float4 *>(p + f);
    const float4 b = *reinterpret_cast<const float4 *>(p + col_up + f);
    gt.x += a.x; gt.y += a.y; gt.z += a.z; gt.w += a.w;
    up.x += b.x; up.y += b.y; up.z += b.z; up.w += b.w;
  }
  auto act = [](float gv, float uv) { return gv / (1.0f + __expf(-gv)) * uv; };
  const float y[4] = {act(gt.x, up.x), act(gt.y, up.y), act(gt.z, up.z), act(gt.w, up.w)};
  uint16_t hi[4], lo[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) split_bf16(y[i], hi[i], lo[i]);
  *reinterpret_cast<uint2 *>(t + (int64_t)r * F + f) =
      make_uint2((uint32_t)hi[0] | ((uint32_t)hi[1] << 16), (uint32_t)hi[2] | ((uint32_t)hi[3] << 16));
  *reinterpret_cast<uint2 *>(t_lo + (int64_t)r * F + f) =
      make_uint2((uint32_t)lo[0] | ((uint32_t)lo[1] << 16), (uint32_t)lo[2] | ((uint32_t)lo[3] << 16));
}

void launch_swiglu_finish(const float *part, int n_splits, int rows, int ldp, int col_up, int F,
                          uint16_t *t, uint16_t *t_lo, hipStream_t st) {
  dim3 grid((F / 4 + 255) / 256, rows);
  swiglu_finish_kernel<<<grid, 256, 0, st>>>(part, n_splits, rows, ldp, col_up, F, t, t_lo);
}

// fp32 -> bf16 row conversion (attention output feeding the output projection)
__global__ void to_bf16_kernel(const float *src, int64_t n, uint16_t *dst, uint16_t *dst_lo) {
  int64_t i = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) * 4;
  if (i >= n) return;
  const float4 v = *reinterpret_cast<const float4 *>(src + i);
  const float y[4] = {v.x, v.y, v.z, v.w};
  uint16_t hi[4], lo[4];
#pragma unroll
  for (int k = 0; k < 4; ++k) split_bf16(y[k], hi[k], lo[k]);
  *reinterpret_cast<uint2 *>(dst + i) =
      make_uint2((uint32_t)hi[0] | ((uint32_t)hi[1] << 16), (uint32_t)hi[2] | ((uint32_t)hi[3] << 16));
  *reinterpret_cast<uint2 *>(dst_lo + i) =
      make_uint2((uint32_t)lo[0] | ((uint32_t)lo[1] << 16), (uint32_t)lo[2] | ((uint32_t)lo[3] << 16));
}

void launch_to_bf16(const float *src, int64_t n, uint16_t *dst, uint16_t *dst_lo, hipStream_t st) {
  to_bf16_kernel<<<(unsigned)((n / 4 + 255) / 256), 256, 0, st>>>(src, n, dst, dst_lo);
}

// logits[r][v] = sum_s part[s][r][v]; per-(row, block) best (value, lowest index); optional
// store of the logits into the caller's padded array.  A second tiny kernel merges the blocks.
__global__ __launch_bounds__(256) void logits_argmax_kernel(StepMeta m, const float *part, int n_splits,
                                                            int ldp, int V, int max_nodes,
                                                            float *logits_out, float *blk_val,
                                                            int *blk_idx) {
  __shared__ float bv[4];
  __shared__ int bi[4];
  const int r = blockIdx.y, rows = m.rows;
  const int v0 = (blockIdx.x * 256 + threadIdx.x) * 4;
  float best = -INFINITY;
  int besti = 0x7fffffff;
  if (v0 < V) {
    float4 a = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int s = 0; s < n_splits; ++s) {
      const float4 p = *reinterpret_cast<const float4 *>(part + ((int64_t)s * rows + r) * ldp + v0);
      a.x += p.x; a.y += p.y; a.z += p.z; a.w += p.w;
    }
    const float vals[4] = {a.x, a.y, a.z, a.w};
    if (logits_out) {
      float *dst = logits_out + ((int64_t)m.seq[r] * max_nodes + m.node[r]) * V + v0;
      for (int i = 0; i < 4; ++i)
        if (v0 + i < V) dst[i] = vals[i];
    }
    for (int i = 0; i < 4; ++i)
      if (v0 + i < V && vals[i] > best) { best = vals[i]; besti = v0 + i; }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const float ov = __shfl_xor(best, o, 64);
    const int oi = __shfl_xor(besti, o, 64);
    if (ov > best || (ov == best && oi < besti)) { best = ov; besti = oi; }
  }
  if ((threadIdx.x & 63) == 0) { bv[threadIdx.x >> 6] = best; bi[threadIdx.x >> 6] = besti; }
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int w = 1; w < 4; ++w)
      if (bv[w] > best || (bv[w] == best && bi[w] < besti)) { best = bv[w]; besti = bi[w]; }
    blk_val[(int64_t)r * gridDim.x + blockIdx.x] = best;
    blk_idx[(int64_t)r * gridDim.x + blockIdx.x] = besti;
  }
}

__global__ __launch_bounds__(64) void argmax_merge_kernel(StepMeta m, const float *blk_val,
                                                          const int *blk_idx, int n_blk,
                                                          int max_nodes, int32_t *argmax) {
  const int r = blockIdx.x;
  float best = -INFINITY;
  int besti = 0x7fffffff;
  for (int b = threadIdx.x; b < n_blk; b += 64) {
    const float v = blk_val[(int64_t)r * n_blk + b];
    const int i = blk_idx[(int64_t)r * n_blk + b];
    if (v > best || (v == best && i < besti)) { best = v; besti = i; }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const float ov = __shfl_xor(best, o, 64);
    const int oi = __shfl_xor(besti, o, 64);
    if (ov > best || (ov == best && oi < besti)) { best = ov; besti = oi; }
  }
  if (threadIdx.x == 0) argmax[m.seq[r] * max_nodes + m.node[r]] = besti == 0x7fffffff ? 0 : besti;
}

int logits_argmax_blocks(int V) { return ((V + 3) / 4 + 255) / 256; }

void launch_logits_argmax(const StepMeta &m, const float *part, int n_splits, int ldp, int V,
                          int max_nodes, float *logits_out, float *blk_val, int *blk_idx,
                          int32_t *argmax, hipStream_t st) {
  const int n_blk = logits_argmax_blocks(V);
  dim3 grid(n_blk, m.rows);
  logits_argmax_kernel<<<grid, 256, 0, st>>>(m, part, n_splits, ldp, V, max_nodes, logits_out, blk_val, blk_idx);
  argmax_merge_kernel<<<m.rows, 64, 0, st>>>(m, blk_val, blk_idx, n_blk, max_nodes, argmax);
}

}  // namespace specasr
