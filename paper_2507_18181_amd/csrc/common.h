// Shared device helpers and internal layouts of the tree-verification library (gfx950).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace specasr {

constexpr int kWave = 64;

// ---- storage types -------------------------------------------------------
struct bf16_t {
  uint16_t bits;
};

__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ float to_f32(bf16_t v) { return __uint_as_float(((uint32_t)v.bits) << 16); }
__device__ __forceinline__ float bf16_bits_to_f32(uint32_t b) { return __uint_as_float(b << 16); }

// float -> bf16, round to nearest even (finite inputs; NaN keeps a quiet-NaN pattern)
__device__ __forceinline__ uint16_t f32_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

// v = hi + lo with both parts bf16: the pair carries 16 mantissa bits of v
__device__ __forceinline__ void split_bf16(float v, uint16_t &hi, uint16_t &lo) {
  hi = f32_to_bf16_bits(v);
  lo = f32_to_bf16_bits(v - __uint_as_float(((uint32_t)hi) << 16));
}

template <class T> __device__ __forceinline__ T from_f32(float f);
template <> __device__ __forceinline__ float from_f32<float>(float f) { return f; }
template <> __device__ __forceinline__ bf16_t from_f32<bf16_t>(float f) {
  bf16_t r;
  r.bits = f32_to_bf16_bits(f);
  return r;
}

// Element offset of activation (row, col) inside one plane of a B-operand-packed buffer:
// [kstep = col/16][node group = row/32][lane = row%32 + 32*((col%16)/8)][col%8]
__host__ __device__ __forceinline__ int64_t packed_act_offset(int row, int col, int nb) {
  return ((((int64_t)(col >> 4) * nb + (row >> 5)) * 64 + (row & 31) + 32 * ((col >> 3) & 1)) << 3) + (col & 7);
}

// Element offset of split-k partial sum (split s, activation row, output column) in the partial-sum
// buffer: [split][band = col/32][row, padded to rows_pad = 32 or a multiple of 64][col%32].  One (split, band)
// block is contiguous, so the GEMM writes it with full-line stores and a consumer thread reads
// 4 consecutive columns as one float4 (col a multiple of 4).
__host__ __device__ __forceinline__ int64_t part_offset(int s, int row, int col, int n_bands, int rows_pad) {
  return ((((int64_t)s * n_bands + (col >> 5)) * rows_pad + row) << 5) + (col & 31);
}
__host__ __device__ __forceinline__ int part_rows_pad(int rows) { return rows <= 32 ? 32 : (rows + 63) / 64 * 64; }

// ---- per-call tree metadata as the kernels see it ------------------------
// Rows are the tree nodes of all sequences of the call, flattened without
// padding: row = row_start[seq] + node.
struct StepMeta {
  const int32_t *token;      // [rows] token id (ignored where use_embed)
  const int32_t *seq;        // [rows] sequence of the row
  const int32_t *node;       // [rows] node index inside its tree
  const int32_t *depth;      // [rows]
  const int32_t *pos;        // [rows] kv_len[seq] + depth  (rotary position)
  const int32_t *slot;       // [rows] kv_len[seq] + node   (cache slot)
  const int32_t *parent;     // [rows] parent node index inside the tree, -1 for the root
  const int32_t *use_embed;  // [rows]
  const uint64_t *anc;       // [rows] bit j set iff node j is on the row's root path (self included)
  const int32_t *kv_len;     // [batch]
  const int32_t *row_start;  // [batch]
  const int32_t *n_nodes;    // [batch]
  int32_t rows, batch;
  // Copies of kv_len[0] and n_nodes[0] that travel with the kernel arguments: a single-sequence
  // call (the common case) needs no dependent global load to find its key range.
  int32_t kv_len0, n_nodes0;
  __device__ __forceinline__ int seq_of_row(int r) const { return batch == 1 ? 0 : seq[r]; }
  __device__ __forceinline__ int seq_kv_len(int s) const { return batch == 1 ? kv_len0 : kv_len[s]; }
  __device__ __forceinline__ int seq_n_nodes(int s) const { return batch == 1 ? n_nodes0 : n_nodes[s]; }
  __device__ __forceinline__ int seq_row_start(int s) const { return batch == 1 ? 0 : row_start[s]; }
};

// KV cache geometry: element index of (seq, layer, kv head, slot, 0)
struct KvGeom {
  int64_t capacity;
  int32_t n_layers, n_kv_heads, head_dim;
  // 1: every sequence of the call is a window onto the cache of sequence 0 (a long chain cut into
  // pieces that are processed together: piece j is "sequence" j with its own kv_len)
  int32_t shared_cache = 0;
  __host__ __device__ int64_t row(int32_t seq, int32_t layer, int32_t h, int64_t slot) const {
    return ((((int64_t)(shared_cache ? 0 : seq) * n_layers + layer) * n_kv_heads + h) * capacity + slot) * head_dim;
  }
};

// ---- wavefront / block reductions ---------------------------------------
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

// Block-wide reductions for blockDim.x a multiple of 64 and <= 1024. `red` holds >= 16 floats.
__device__ __forceinline__ float block_sum(float v, float *red) {
  v = wave_sum(v);
  const int w = threadIdx.x >> 6, nw = blockDim.x >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[w] = v;
  __syncthreads();
  float t = 0.f;
  for (int i = 0; i < nw; ++i) t += red[i];
  return t;
}
__device__ __forceinline__ float block_max(float v, float *red) {
  v = wave_max(v);
  const int w = threadIdx.x >> 6, nw = blockDim.x >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[w] = v;
  __syncthreads();
  float t = red[0];
  for (int i = 1; i < nw; ++i) t = fmaxf(t, red[i]);
  return t;
}

// Per-row RMSNorm statistics left by launch_residual_gain for the consumer of the next GEMM.
struct RowNorm {
  const float *ssq;  // [rows][n_slab] sums of squares of the residual row, one per column slab
  int n_slab;
  int d;      // row length
  float eps;  // added to the mean square inside the root
};
// 1 / rms of residual row r from the slab sums of squares (eps inside the root, Sec. II-A's decoder
// block), in two steps so that a kernel can have its own loads in flight together with these:
// row_ssq_lane issues the loads of this lane's share (up to 4 at once) and adds them up;
// row_rms_finish sums over the wavefront.  Every lane of the calling wavefront must be active in
// row_rms_finish; all lanes get the same value.
__device__ __forceinline__ float row_ssq_lane(const RowNorm &nrm, int r) {
  const float *p = nrm.ssq + (int64_t)r * nrm.n_slab;
  const int i = threadIdx.x & 63, n = nrm.n_slab;
  const float v0 = i < n ? p[i] : 0.f, v1 = i + 64 < n ? p[i + 64] : 0.f;
  const float v2 = i + 128 < n ? p[i + 128] : 0.f, v3 = i + 192 < n ? p[i + 192] : 0.f;
  float s = (v0 + v1) + (v2 + v3);
  for (int k = i + 256; k < n; k += 64) s += p[k];
  return s;
}
__device__ __forceinline__ float row_rms_finish(const RowNorm &nrm, float lane_ssq) {
  return 1.0f / sqrtf(wave_sum(lane_ssq) / (float)nrm.d + nrm.eps);
}
__device__ __forceinline__ float row_rms_scale(const RowNorm &nrm, int r) {
  return row_rms_finish(nrm, row_ssq_lane(nrm, r));
}

}  // namespace specasr
