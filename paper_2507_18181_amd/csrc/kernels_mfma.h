// Launchers of the bf16 MFMA stages (see kernels_mfma.hip).
#pragma once
#include "kernels.h"

namespace specasr {


// A weight matrix repacked into MFMA A-operand tiles: [n_bands][ksteps][64 lanes][8 bf16].
struct PackedMatrix {
  void *data = nullptr;
  int n_bands = 0;  // bands of 32 output features (last one zero padded)
  int ksteps = 0;   // in_features / 16
  int ldo = 0;      // n_bands * 32: row stride of the partial-sum output
};

struct GemmPlan {
  int n_splits = 1;  // k-chunks across workgroups (partial sums per output)
  int lw = 16;       // ring slots per wavefront: >= its k-slice, one of the instantiated sizes
  int grid = 256;    // workgroups, a multiple of n_splits (one per compute unit)
  bool wide = false; // many rows: the tiled kernel (only n_splits applies)
};

void launch_read_probe(const void *buf, size_t bytes, int grid, uint32_t *sink, hipStream_t st);
void launch_repack(const void *src, int n_out, int K, void *dst, int band0, hipStream_t st);
hipError_t gemm_skinny_set_lds_limit();
void launch_gemm_skinny(const PackedMatrix &W, const uint16_t *Xp, int rows, float *part,
                        const GemmPlan &plan, int stage, hipStream_t st,
                        hipEvent_t ev0 = nullptr, hipEvent_t ev1 = nullptr);
// large row counts (prefill): rows padded to workgroup tiles of 128, in groups of 32
int wide_row_groups(int rows);
int wide_gemm_splits(int n_bands, int ksteps, int rows, int n_cu);
void launch_gemm_wide(const PackedMatrix &W, const uint16_t *Xp, int rows, float *part, int n_splits,
                      int stage, hipStream_t st, hipEvent_t ev0 = nullptr, hipEvent_t ev1 = nullptr);
int residual_slabs(int d);
void launch_residual_gain(float *x, const float *part, int n_splits, int rows, int ldp,
                          const void *gain, int d, uint16_t *hb, uint16_t *hb_lo, int nb, float *ssq,
                          hipStream_t st, int rows_pad = 0);
void launch_qkv_finish(const StepMeta &m, const ModelDims &md, const KvGeom &g, int layer,
                       const float *part, int n_splits, int ldp, const RowNorm &nrm, int col_k,
                       int col_v, const float2 *cs, float *q, uint16_t *qb, uint16_t *qb_lo, void *kc,
                       void *vc, hipStream_t st);
void launch_swiglu_finish(const float *part, int n_splits, int rows, int ldp, const RowNorm &nrm,
                          int col_up, int F, uint16_t *t, uint16_t *t_lo, int nb, hipStream_t st);
void launch_to_bf16(const float *src, int rows, int K, uint16_t *dst, uint16_t *dst_lo, hipStream_t st);
int logits_argmax_blocks(int V);
void launch_logits_argmax(const StepMeta &m, const float *part, int n_splits, int ldp,
                          const RowNorm &nrm, int V, int max_nodes, float *logits_out, float *blk_val, int *blk_idx,
                          int32_t *argmax, hipStream_t st);

// tree-masked MFMA attention (kernels_attn.hip)
bool tree_attention_supported(int head_dim);
int tree_attention_max_chunks(int n_kv_heads);
hipError_t tree_attention_set_lds_limit();
void launch_tree_attention(const StepMeta &m, const ModelDims &md, const KvGeom &g, int layer,
                           int max_total_keys, int max_seq_nodes, const uint16_t *qb,
                           const uint16_t *qb_lo, const void *kc, const void *vc, float *o_part,
                           float *ml_part, uint16_t *out, uint16_t *out_lo, int nb, int min_chunk_keys,
                           hipStream_t st);

}  // namespace specasr
