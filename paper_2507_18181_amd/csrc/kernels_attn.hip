// Tree-masked attention for gfx950 with bf16 MFMA (Sec. II-B: 2D attention mask over the draft
// token tree; Sec. IV-C: used to verify the two-pass sparse tree).
//
// Every tree node attends to the cached prefix [0, kv_len) and to the cache slots of the nodes
// on its own root path.  The KV cache is streamed exactly once per KV head: one wavefront takes
// (sequence, KV head, chunk of keys) and serves ALL query rows that share the head (the
// grouped-query heads times the tree nodes), 32 queries per MFMA column block.
//
//   S^T[key][query] = K[key][:] . Q[query][:]      A = K tile (rows = keys, read straight from
//                                                   the cache, 16 B per lane), B = Q^T
//   online softmax per query column (fp32; max and sum via one cross-half shuffle)
//   Q and P enter the matrix cores as hi + lo bf16 planes (two MFMAs), so only the bf16 storage
//   of the cache itself limits the precision.
//   O^T[c][query]  += V^T[c][key] * P^T[key][query] A = V^T gathered from an LDS copy of the V
//                                                   tile with key pairs interleaved, B = P^T,
//                                                   which is exactly how the lanes already hold P
//
// Partial (unnormalised) outputs per key chunk are merged by a second small kernel.
#include "kernels.h"
#include "kernels_mfma.h"

namespace specasr {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  return (uint32_t)f32_to_bf16_bits(lo) | ((uint32_t)f32_to_bf16_bits(hi) << 16);
}

// Two finite floats -> their hi planes packed (a in the low half) and their lo planes packed, with
// the hardware's round-to-nearest-even conversion (one v_cvt_pk_bf16_f32 per pair and plane; the
// same values as split_bf16 for the probabilities this is used on).
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) float f32x2;
__device__ __forceinline__ void split_bf16_pair(float a, float b, uint32_t &hi, uint32_t &lo) {
  const bf16x2 h = __builtin_convertvector((f32x2){a, b}, bf16x2);
  hi = __builtin_bit_cast(uint32_t, h);
  const float ra = a - __uint_as_float(hi << 16), rb = b - __uint_as_float(hi & 0xffff0000u);
  const bf16x2 l = __builtin_convertvector((f32x2){ra, rb}, bf16x2);
  lo = __builtin_bit_cast(uint32_t, l);
}

// grid (8 * n_rgb * ceil(n_chunks * Hkv / 8), 1, batch), block 256.  Workgroups go to the 8 XCDs
// round-robin by their linear index, so the n_rgb workgroups that stream the SAME keys for
// different query row groups are placed 8 apart: they run on one XCD and share its L2.
// Block 256: the four wavefronts of a workgroup take the
// 32-key tiles of the chunk round-robin, each with its own online softmax, and merge their
// (max, sum, output) through LDS into ONE partial result per chunk.  RGW = query row groups (of
// 32) per workgroup.
template <int HD, int RGW>
__global__ __launch_bounds__(256) void tree_attention_kernel(StepMeta m, KvGeom g, int layer, int H,
                                                            int Hkv, int n_rgb,
                                                            const uint16_t *__restrict__ qb,
                                                            const uint16_t *__restrict__ qb_lo,
                                                            const uint16_t *__restrict__ kc,
                                                            const uint16_t *__restrict__ vc,
                                                            int chunk_keys, int n_chunks,
                                                            float *__restrict__ o_part,
                                                            float *__restrict__ ml_part,
                                                            uint16_t *__restrict__ out,
                                                            uint16_t *__restrict__ out_lo, int nb) {
  constexpr int KK = HD / 16;  // MFMA k-steps across the head dimension
  constexpr int CB = HD / 32;  // 32-wide output column blocks
  // LDS: per wavefront two V tiles [key pair][column] (low half = even key); reused afterwards
  // for the cross-wavefront merge: o[wave][rg][cb][j][lane] floats, then (m, l)[wave][rg][32]
  extern __shared__ uint32_t lds_attn[];
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  uint32_t *vp = lds_attn + wave * (2 * 16 * HD);
  const int lane = threadIdx.x & 63, h = lane >> 5, ql = lane & 31;
  const int rgb = (blockIdx.x >> 3) % n_rgb, base = ((blockIdx.x >> 3) / n_rgb) * 8 + (blockIdx.x & 7);
  if (base >= n_chunks * Hkv) return;
  // Sequences are dispatched last to first: the pieces of a prefill pass come in order of growing
  // key count, and the workgroups with the longest key loops should start first.
  const int chunk = base % n_chunks, kvh = base / n_chunks, seq = gridDim.z - 1 - blockIdx.z;
  const int G = H / Hkv;
  const int L = m.seq_kv_len(seq), n = m.seq_n_nodes(seq), r0 = m.seq_row_start(seq), rows = m.rows;
  const int T = L + n, QR = G * n;
  const int t_begin = chunk * chunk_keys;
  if (t_begin >= T || rgb * RGW * 32 >= QR) return;
  const int t_end = min(T, t_begin + chunk_keys);

  // queries of this wavefront
  bool valid[RGW];
  int out_row[RGW], out_head[RGW];
  uint64_t anc[RGW];
  u32x4 qreg[RGW][KK], qlo[RGW][KK];  // queries as hi + lo bf16 planes
#pragma unroll
  for (int w = 0; w < RGW; ++w) {
    const int qrow = (rgb * RGW + w) * 32 + ql;
    valid[w] = qrow < QR;
    const int gi = valid[w] ? qrow / n : 0, node = valid[w] ? qrow - gi * n : 0;
    out_row[w] = r0 + node;
    out_head[w] = kvh * G + gi;
    anc[w] = valid[w] ? m.anc[out_row[w]] : 0ull;
    const int64_t qoff = ((int64_t)out_row[w] * H + out_head[w]) * HD + 8 * h;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      qreg[w][kk] = valid[w] ? *reinterpret_cast<const u32x4 *>(qb + qoff + 16 * kk) : (u32x4){0u, 0u, 0u, 0u};
      qlo[w][kk] = valid[w] ? *reinterpret_cast<const u32x4 *>(qb_lo + qoff + 16 * kk) : (u32x4){0u, 0u, 0u, 0u};
    }
  }
  float m_run[RGW], l_run[RGW];
  f32x16 o[RGW][CB];
#pragma unroll
  for (int w = 0; w < RGW; ++w) {
    m_run[w] = -INFINITY;
    l_run[w] = 0.f;
#pragma unroll
    for (int cb = 0; cb < CB; ++cb)
#pragma unroll
      for (int j = 0; j < 16; ++j) o[w][cb][j] = 0.f;
  }
  const uint16_t *kbase = kc + g.row(seq, layer, kvh, 0);
  const uint16_t *vbase = vc + g.row(seq, layer, kvh, 0);

  // One register set for the tile in flight: K as A-operand registers, V as raw row pairs that are
  // interleaved into LDS when consumed.  Each half is requested again for the wavefront's NEXT
  // tile as soon as the current tile has consumed it (V after its copy to LDS, K after the last
  // QK^T product), so the loads have the rest of the tile's work to arrive -- and the kernel keeps
  // one tile's worth of staging registers instead of two.
  constexpr int VI = HD / 32;  // (key pair, 8-column group) items per lane
  u32x4 kreg[KK], va[VI], vb[VI];
  auto issue_k = [&](int t0) {
    const uint16_t *kp = kbase + (int64_t)min(t0 + ql, T - 1) * HD + 8 * h;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) kreg[kk] = *reinterpret_cast<const u32x4 *>(kp + 16 * kk);
  };
  auto issue_v = [&](int t0) {
#pragma unroll
    for (int x = 0; x < VI; ++x) {
      const int it = lane + 64 * x;
      const int pair = it / (HD / 8), cg = it - pair * (HD / 8);
      const int k0 = min(t0 + 2 * pair, T - 1), k1 = min(t0 + 2 * pair + 1, T - 1);
      va[x] = *reinterpret_cast<const u32x4 *>(vbase + (int64_t)k0 * HD + 8 * cg);
      vb[x] = *reinterpret_cast<const u32x4 *>(vbase + (int64_t)k1 * HD + 8 * cg);
    }
  };
  auto compute = [&](int t0, uint32_t *vpb, bool more) {
    // V tile into LDS, two keys interleaved per 32-bit word (low half = even key)
#pragma unroll
    for (int x = 0; x < VI; ++x) {
      const int it = lane + 64 * x;
      const int pair = it / (HD / 8), cg = it - pair * (HD / 8);
      const u32x4 a = va[x], b = vb[x];
      u32x4 lo, hi;  // columns 8cg..8cg+3 and 8cg+4..8cg+7
      lo[0] = (a[0] & 0xffffu) | (b[0] << 16);
      lo[1] = (a[0] >> 16) | (b[0] & 0xffff0000u);
      lo[2] = (a[1] & 0xffffu) | (b[1] << 16);
      lo[3] = (a[1] >> 16) | (b[1] & 0xffff0000u);
      hi[0] = (a[2] & 0xffffu) | (b[2] << 16);
      hi[1] = (a[2] >> 16) | (b[2] & 0xffff0000u);
      hi[2] = (a[3] & 0xffffu) | (b[3] << 16);
      hi[3] = (a[3] >> 16) | (b[3] & 0xffff0000u);
      u32x4 *dst = reinterpret_cast<u32x4 *>(vpb + pair * HD + 8 * cg);
      dst[0] = lo;
      dst[1] = hi;
    }
    // only this wavefront reads the tile back: its own LDS operations stay in program order
    __builtin_amdgcn_wave_barrier();
    if (more) issue_v(t0 + 128);
#pragma unroll
    for (int w = 0; w < RGW; ++w) {
      f32x16 sT, sT2;  // hi and lo query planes on separate accumulators (independent chains)
#pragma unroll
      for (int j = 0; j < 16; ++j) { sT[j] = 0.f; sT2[j] = 0.f; }
#pragma unroll
      for (int kk = 0; kk < KK; ++kk) {
        sT = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, kreg[kk]),
                                                     __builtin_bit_cast(bf16x8, qreg[w][kk]), sT, 0, 0, 0);
        sT2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, kreg[kk]),
                                                      __builtin_bit_cast(bf16x8, qlo[w][kk]), sT2, 0, 0, 0);
      }
      if (w == RGW - 1 && more) issue_k(t0 + 128);
      // lane holds, for query ql, the keys t0 + 8*(j/4) + 4*h + j%4
      float mx = -INFINITY;
      if (t0 + 32 <= L) {  // tile inside the prefix: every key visible to every valid query
#pragma unroll
        for (int j = 0; j < 16; ++j) {
          sT[j] = valid[w] ? sT[j] + sT2[j] : -INFINITY;
          mx = fmaxf(mx, sT[j]);
        }
      } else {
#pragma unroll
        for (int j = 0; j < 16; ++j) {
          const int key = t0 + 8 * (j >> 2) + 4 * h + (j & 3);
          const bool vis = valid[w] && key < T && (key < L || ((anc[w] >> ((key - L) & 63)) & 1ull));
          sT[j] = vis ? sT[j] + sT2[j] : -INFINITY;
          mx = fmaxf(mx, sT[j]);
        }
      }
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
      const float m_new = fmaxf(m_run[w], mx);
      const bool any = m_new != -INFINITY;
      const float alpha = (m_run[w] == -INFINITY) ? 0.f : __expf(m_run[w] - m_new);
      // exp(-inf) = 0 covers the masked keys; a query that has seen no key yet (m_new = -inf)
      // subtracts 0 instead, so that all of its scores stay -inf and give 0 as well
      const float m_sub = any ? m_new : 0.f;
      float p[16], psum = 0.f;
#pragma unroll
      for (int j = 0; j < 16; ++j) {
        p[j] = __expf(sT[j] - m_sub);
        psum += p[j];
      }
      psum += __shfl_xor(psum, 32, 64);
      const bool rescale = alpha != 1.0f && l_run[w] != 0.f;  // something accumulated and the max moved
      l_run[w] = l_run[w] * alpha + psum;
      m_run[w] = m_new;
      if (__ballot(rescale) != 0ull) {
#pragma unroll
        for (int cb = 0; cb < CB; ++cb)
#pragma unroll
          for (int j = 0; j < 16; ++j) o[w][cb][j] *= alpha;
      }
      // P^T as B operand: MFMA mm covers keys 16*mm .. 16*mm+15 of the tile; this lane's k-slots
      // i = 0..7 are keys 16*mm + 8*(i/4) + 4*h + i%4, i.e. its own p[8*mm + i]
#pragma unroll
      for (int mm = 0; mm < 2; ++mm) {
        u32x4 pb, pl;  // probabilities as hi + lo bf16 planes
#pragma unroll
        for (int i2 = 0; i2 < 4; ++i2) {
          uint32_t hi2, lo2;
          split_bf16_pair(p[8 * mm + 2 * i2], p[8 * mm + 2 * i2 + 1], hi2, lo2);
          pb[i2] = hi2;
          pl[i2] = lo2;
        }
        // matching V^T k-slots: key pairs 8*mm + 2*h, +1, 8*mm + 4 + 2*h, +1
        const uint32_t *vrow = vpb + (8 * mm + 2 * h) * HD + ql;
#pragma unroll
        for (int cb = 0; cb < CB; ++cb) {
          u32x4 vreg;
          vreg[0] = vrow[32 * cb];
          vreg[1] = vrow[32 * cb + HD];
          vreg[2] = vrow[32 * cb + 4 * HD];
          vreg[3] = vrow[32 * cb + 5 * HD];
          o[w][cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, vreg),
                                                             __builtin_bit_cast(bf16x8, pb), o[w][cb], 0, 0, 0);
          o[w][cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, vreg),
                                                             __builtin_bit_cast(bf16x8, pl), o[w][cb], 0, 0, 0);
        }
      }
    }
  };

  const int t_first = t_begin + 32 * wave;  // this wavefront's tiles: t_first, +128, +256, ...
  if (t_first < t_end) {
    issue_k(t_first);
    issue_v(t_first);
  }
  int vbuf = 0;  // the two LDS tiles of the wavefront alternate
  for (int t0 = t_first; t0 < t_end; t0 += 128, vbuf ^= 1) compute(t0, vp + vbuf * (16 * HD), t0 + 128 < t_end);

  // merge the four wavefronts: everything to LDS in register layout, then wavefront cb reduces
  // column block cb and writes the workgroup's partial result
  __syncthreads();
  float *lo_ = reinterpret_cast<float *>(lds_attn);
  float *lml = lo_ + 4 * RGW * CB * 1024;
#pragma unroll
  for (int w = 0; w < RGW; ++w) {
#pragma unroll
    for (int cb = 0; cb < CB; ++cb)
#pragma unroll
      for (int j = 0; j < 16; ++j) lo_[(((wave * RGW + w) * CB + cb) * 16 + j) * 64 + lane] = o[w][cb][j];
    if (h == 0) {
      lml[((wave * RGW + w) * 32 + ql) * 2] = m_run[w];
      lml[((wave * RGW + w) * 32 + ql) * 2 + 1] = l_run[w];
    }
  }
  __syncthreads();
  if (wave < CB) {
    const int cb = wave;
#pragma unroll
    for (int w = 0; w < RGW; ++w) {
      float mw[4], M = -INFINITY;
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        mw[v] = lml[((v * RGW + w) * 32 + ql) * 2];
        M = fmaxf(M, mw[v]);
      }
      float Lsum = 0.f, acc[16];
#pragma unroll
      for (int j = 0; j < 16; ++j) acc[j] = 0.f;
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const float wgt = (mw[v] == -INFINITY) ? 0.f : __expf(mw[v] - M);
        Lsum += wgt * lml[((v * RGW + w) * 32 + ql) * 2 + 1];
#pragma unroll
        for (int j = 0; j < 16; ++j) acc[j] += wgt * lo_[(((v * RGW + w) * CB + cb) * 16 + j) * 64 + lane];
      }
      if (!valid[w]) continue;
      // O^T lane layout = query column ql, output columns 32*cb + 8*(j/4) + 4*h + j%4
      if (out != nullptr) {
        // every sequence is a single chunk: this IS the result -- normalise and write the packed
        // hi/lo planes the output projection reads (what the merge kernel would do with one chunk)
        const int col0 = out_head[w] * HD + 32 * cb + 4 * h;
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          uint16_t hi4[4], lo4[4];
#pragma unroll
          for (int i = 0; i < 4; ++i) split_bf16(acc[4 * q4 + i] / Lsum, hi4[i], lo4[i]);
          const int64_t po = packed_act_offset(out_row[w], col0 + 8 * q4, nb);
          *reinterpret_cast<uint2 *>(out + po) =
              make_uint2((uint32_t)hi4[0] | ((uint32_t)hi4[1] << 16), (uint32_t)hi4[2] | ((uint32_t)hi4[3] << 16));
          *reinterpret_cast<uint2 *>(out_lo + po) =
              make_uint2((uint32_t)lo4[0] | ((uint32_t)lo4[1] << 16), (uint32_t)lo4[2] | ((uint32_t)lo4[3] << 16));
        }
        continue;
      }
      const int64_t base = ((int64_t)chunk * rows + out_row[w]) * H + out_head[w];
      float *op = o_part + base * HD + 32 * cb + 4 * h;
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4)
        *reinterpret_cast<float4 *>(op + 8 * q4) = make_float4(acc[4 * q4], acc[4 * q4 + 1], acc[4 * q4 + 2], acc[4 * q4 + 3]);
      if (cb == 0 && h == 0) {
        ml_part[base * 2] = M;
        ml_part[base * 2 + 1] = Lsum;
      }
    }
  }
}

// Merge the key chunks: out = sum_c e^(m_c - M) o_c / sum_c e^(m_c - M) l_c, rounded to bf16.
// grid (H, rows), block HD.
__global__ void tree_attention_merge_kernel(StepMeta m, int H, int HD, int chunk_keys,
                                            const float *__restrict__ o_part,
                                            const float *__restrict__ ml_part,
                                            uint16_t *__restrict__ out, uint16_t *__restrict__ out_lo,
                                            int nb) {
  const int a = blockIdx.x, r = blockIdx.y, c = threadIdx.x, rows = m.rows;
  const int seq = m.seq_of_row(r);
  const int T = m.seq_kv_len(seq) + m.seq_n_nodes(seq);
  const int n_chunks = (T + chunk_keys - 1) / chunk_keys;
  // batches of 8 chunks with all loads issued together; running (max, numerator, denominator)
  float M = -INFINITY, num = 0.f, den = 0.f;
  const int64_t cstride = (int64_t)rows * H;
  const int64_t base0 = (int64_t)r * H + a;
  for (int c0 = 0; c0 < n_chunks; c0 += 8) {
    float mc[8], lc[8], oc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int ch = min(c0 + i, n_chunks - 1);
      const int64_t base = base0 + ch * cstride;
      mc[i] = (c0 + i < n_chunks) ? ml_part[base * 2] : -INFINITY;
      lc[i] = ml_part[base * 2 + 1];
      oc[i] = o_part[base * HD + c];
    }
    float Mb = M;
#pragma unroll
    for (int i = 0; i < 8; ++i) Mb = fmaxf(Mb, mc[i]);
    if (Mb == -INFINITY) continue;
    const float scale = (M == -INFINITY) ? 0.f : __expf(M - Mb);
    num *= scale;
    den *= scale;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const float wgt = (mc[i] == -INFINITY) ? 0.f : __expf(mc[i] - Mb);
      num += wgt * oc[i];
      den += wgt * lc[i];
    }
    M = Mb;
  }
  const int64_t oi = packed_act_offset(r, a * HD + c, nb);  // B-operand order of the output projection
  split_bf16(num / den, out[oi], out_lo[oi]);
}

template <int HD>
static void launch_attn_hd(const StepMeta &m, const ModelDims &md, const KvGeom &g, int layer,
                           int max_seq_nodes, int chunk_keys, int n_chunks,
                           const uint16_t *qb, const uint16_t *qb_lo, const void *kc, const void *vc,
                           float *o_part, float *ml_part, uint16_t *out, uint16_t *out_lo, int nb,
                           hipStream_t st) {
  const int G = md.n_heads / md.n_kv_heads;
  const int row_groups = (G * max_seq_nodes + 31) / 32;
  const bool direct = n_chunks == 1;  // nothing to merge: the attention kernel writes the final planes
  // LDS: 4 wavefronts x 2 V tiles, reused for the merge (4 x RGW x HD/32 x 4 KB + (m, l))
  auto lds_bytes = [](int rgw) {
    const size_t vt = (size_t)4 * 2 * 16 * HD * 4;
    const size_t mg = (size_t)4 * rgw * (HD / 32) * 4096 + (size_t)4 * rgw * 32 * 2 * 4;
    return vt > mg ? vt : mg;
  };
  dim3 grid((n_chunks * md.n_kv_heads + 7) / 8 * 8 * row_groups, 1, m.batch);
  tree_attention_kernel<HD, 1><<<grid, 256, lds_bytes(1), st>>>(m, g, layer, md.n_heads, md.n_kv_heads, row_groups, qb, qb_lo, (const uint16_t *)kc, (const uint16_t *)vc, chunk_keys, n_chunks, o_part, ml_part, direct ? out : nullptr, direct ? out_lo : nullptr, nb);
  if (direct) return;
  dim3 mgrid(md.n_heads, m.rows);
  tree_attention_merge_kernel<<<mgrid, HD, 0, st>>>(m, md.n_heads, HD, chunk_keys, o_part, ml_part, out, out_lo, nb);
}

bool tree_attention_supported(int head_dim) { return head_dim == 64 || head_dim == 128; }

int tree_attention_max_chunks(int n_kv_heads) { return 256 / n_kv_heads + 2; }

hipError_t tree_attention_set_lds_limit() {
  const int big = 4 * 4 * 4096 + 4 * 32 * 2 * 4;  // merge area at head_dim 128: the larger of the two uses
  hipError_t e = hipFuncSetAttribute((const void *)tree_attention_kernel<128, 1>, hipFuncAttributeMaxDynamicSharedMemorySize, big);
  if (e != hipSuccess) return e;
  return hipFuncSetAttribute((const void *)tree_attention_kernel<64, 1>, hipFuncAttributeMaxDynamicSharedMemorySize, big);
}

// Key-chunk size (a multiple of 32).  One sequence: ~256 workgroups (one per compute unit) over
// its keys.  Several sequences (a batch, or the pieces of a wide prefill pass): if (KV heads x
// sequences x row-group blocks) already gives a workgroup per compute unit, every sequence is one
// chunk (measured on the 7B prefill: 23.7 us against 28.8 with two chunks); otherwise the sequences
// differ in length and there are few heads to spread them, so the chunks are made smaller -- ~1024
// workgroups if all were as long as the longest, at least 128 keys (one tile per wavefront) -- and
// the short ones simply need fewer of them (1.1B, 16 utterances: 67 us against 80); the number of
// chunks stays within what the wide workspace holds (128 / n_kv_heads + 1).
int tree_attention_chunk_keys(int max_total_keys, int n_kv_heads, int batch, int row_group_blocks, int min_chunk_keys) {
  const long target = batch > 1 ? 1024 : 256;
  long want = ((long)max_total_keys * n_kv_heads * batch * row_group_blocks + target - 1) / target;
  long ck = (want + 31) / 32 * 32;
  if (ck < 32) ck = 32;
  // a short single sequence: one chunk, the attention kernel writes the result itself and no merge
  // kernel runs (1.1B, ~360 keys: 1.536 against 1.555 ms per forward; at 842 keys it loses)
  if (batch == 1 && max_total_keys <= 512) ck = 512;
  if (batch > 1) {
    if (ck < 128) ck = 128;
    if ((long)n_kv_heads * batch * row_group_blocks >= 256) ck = ((long)max_total_keys + 31) / 32 * 32;
    const long max_chunks = 128 / n_kv_heads + 1;
    const long ck_min = ((max_total_keys + max_chunks - 1) / max_chunks + 31) / 32 * 32;
    if (ck < ck_min) ck = ck_min;
  }
  if (min_chunk_keys / 32 * 32 > ck) ck = min_chunk_keys / 32 * 32;  // development aid: never below the automatic size
  return (int)ck;
}

void launch_tree_attention(const StepMeta &m, const ModelDims &md, const KvGeom &g, int layer,
                           int max_total_keys, int max_seq_nodes, const uint16_t *qb,
                           const uint16_t *qb_lo, const void *kc, const void *vc, float *o_part,
                           float *ml_part, uint16_t *out, uint16_t *out_lo, int nb, int min_chunk_keys,
                           hipStream_t st) {
  const int G = md.n_heads / md.n_kv_heads;
  // One query row group (32 rows) per workgroup.  Two per workgroup would halve the key traffic
  // (head_dim 64: the accumulators would fit), but the keys of a head are L2 hits after their
  // first use and the kernel is bound by its softmax arithmetic: measured slower wherever it was
  // tried (16 utterances on the 1.1B model: 43 against 38 us).
  const int row_groups = (G * max_seq_nodes + 31) / 32;
  const int ck = tree_attention_chunk_keys(max_total_keys, md.n_kv_heads, m.batch, row_groups, min_chunk_keys);
  const int n_chunks = (max_total_keys + ck - 1) / ck;
  if (md.head_dim == 64)
    launch_attn_hd<64>(m, md, g, layer, max_seq_nodes, ck, n_chunks, qb, qb_lo, kc, vc, o_part, ml_part, out, out_lo, nb, st);
  else
    launch_attn_hd<128>(m, md, g, layer, max_seq_nodes, ck, n_chunks, qb, qb_lo, kc, vc, o_part, ml_part, out, out_lo, nb, st);
}

}  // namespace specasr
