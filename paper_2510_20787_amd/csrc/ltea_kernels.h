// Host-side launcher declarations: one per kernel family. All pointers are device pointers unless
// stated otherwise; every launcher enqueues on `stream` and returns the hipError_t of the launch.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/ltea.h"

namespace ltea {

struct SeqView {              // packed-token description shared by all prefill launchers
  const int32_t* cu_seqlens;  // device [n_seqs+1]
  int32_t n_seqs;
  int64_t total_tokens;
  int32_t max_seqlen;
};

inline int cnn_rho(const ltea_cnn* c) {
  int r = 0;
  for (int l = 0; l < c->n_layers; ++l) r += c->dilation[l] * (c->kernel[l] - 1) / 2;
  return r;
}

// ---- (a) scoring -------------------------------------------------------------------------------
// The matrix-core scoring kernels address the K/V rows of one workgroup (a group of token tiles plus halo, never
// more than this many rows) with 32-bit byte offsets from a 64-bit base of their own, so a sequence may be of any
// length; only the token stride is bounded.
constexpr int kScoreRowsPerDescriptor = 2304;
inline bool score_stride_ok(int64_t stride_tok) {
  return stride_tok * 2 * kScoreRowsPerDescriptor < ((int64_t)1 << 31);
}
// Generic layered path (any depth, fp32 or bf16 storage, VALU): needs 2 * Hkv * T * max(c_out) floats
// of scratch when n_layers > 1, Hkv * T * c_out[0] floats when n_layers == 1.
size_t score_generic_workspace(const ltea_cfg& cfg, const ltea_cnn& cnn, int64_t total_tokens);
hipError_t launch_score_generic(const ltea_cfg& cfg, const ltea_cnn& cnn, const void* k, const void* v,
                                int64_t stride_tok, int64_t stride_head, const SeqView& sv, float* logits,
                                void* workspace, hipStream_t stream);
// Single-layer bf16 path on MFMA (fused conv + Swish + output projection); the workspace holds the weights
// re-laid as tap-major panels unless cnn.panels supplies them (launch_*_panels writes either).
bool score_mfma_supported(const ltea_cfg& cfg, const ltea_cnn& cnn);
size_t score_mfma_workspace(const ltea_cfg& cfg, const ltea_cnn& cnn);
hipError_t launch_score_mfma_panels(const ltea_cfg& cfg, const ltea_cnn& cnn, void* panels, hipStream_t stream);
hipError_t launch_score_mfma(const ltea_cfg& cfg, const ltea_cnn& cnn, const void* k, const void* v,
                             int64_t stride_tok, int64_t stride_head, const SeqView& sv, float* logits,
                             void* workspace, hipStream_t stream);

// The same layer with the weights held in registers and the tokens loaded straight into LDS (D = 64, kernel 3 or 5).
// Its panels have the same size but are ordered as the registers hold them; launch_score_mfma and
// launch_score_mfma_panels hand over to these where they apply.
bool score_reg_supported(const ltea_cfg& cfg, const ltea_cnn& cnn);
// launch_score_reg with panels == nullptr reads cnn.w[0] as the caller holds it and sorts it inside the kernel;
// that needs the tensor 16-byte aligned.
bool score_reg_takes_raw_weights(const ltea_cnn& cnn);
hipError_t launch_score_reg_panels(const ltea_cfg& cfg, const ltea_cnn& cnn, void* panels, hipStream_t stream);
hipError_t launch_score_reg(const ltea_cfg& cfg, const ltea_cnn& cnn, const void* k, const void* v, int64_t stride_tok,
                            int64_t stride_head, const SeqView& sv, float* logits, const void* panels,
                            hipStream_t stream);

// Multi-layer bf16 path on MFMA (all layers fused, activations in LDS as hi + lo bf16 pairs); the workspace holds
// every layer's weights re-laid as tap-major panels.
// The paper's own stack (D = 64, three kernel-3 layers of 64 / 32 / 16 channels) with every layer's weights held in
// registers and the tokens loaded straight into LDS; its panels have the size of the general kernel's but are ordered
// as the registers hold them.  launch_score_deep and launch_score_deep_panels hand over to these where they apply.
bool score_deep_reg_supported(const ltea_cfg& cfg, const ltea_cnn& cnn);
// launch_score_deep_reg with panels == nullptr reads cnn.w[0..2] as the caller holds them and sorts them inside the
// kernel; that needs the three tensors 16-byte aligned.
bool score_deep_reg_takes_raw_weights(const ltea_cnn& cnn);
hipError_t launch_score_deep_reg_panels(const ltea_cfg& cfg, const ltea_cnn& cnn, void* panels, hipStream_t stream);
// row_valid (optional, device, one byte per token row): windows mode for the decode step.  The rows are many
// independent short windows laid end to end with at least max(dilation) rows of zeros between them; a 0 byte marks a
// row that is not a token, whose activations are then zero at every layer, as outside a sequence.
hipError_t launch_score_deep_reg(const ltea_cfg& cfg, const ltea_cnn& cnn, const void* k, const void* v,
                                 int64_t stride_tok, int64_t stride_head, const SeqView& sv, float* logits,
                                 const void* panels, hipStream_t stream, const uint8_t* row_valid = nullptr);
bool score_deep_supported(const ltea_cfg& cfg, const ltea_cnn& cnn);
size_t score_deep_workspace(const ltea_cfg& cfg, const ltea_cnn& cnn);
hipError_t launch_score_deep_panels(const ltea_cfg& cfg, const ltea_cnn& cnn, void* panels, hipStream_t stream);
hipError_t launch_score_deep(const ltea_cfg& cfg, const ltea_cnn& cnn, const void* k, const void* v,
                             int64_t stride_tok, int64_t stride_head, const SeqView& sv, float* logits,
                             void* workspace, hipStream_t stream, const uint8_t* row_valid = nullptr);

// ---- (b) retention + cache fill -------------------------------------------------------------------
hipError_t launch_retain(const ltea_cfg& cfg, const float* logits, const void* k, const void* v,
                         int64_t stride_tok, int64_t stride_head, const SeqView& sv, int rho,
                         const ltea_cache& cache, hipStream_t stream);

// ---- (c) prefill attention -------------------------------------------------------------------------
hipError_t launch_attention_generic(const ltea_cfg& cfg, const void* q, int64_t q_stride_tok, int64_t q_stride_head,
                                    const void* k, const void* v, int64_t kv_stride_tok, int64_t kv_stride_head,
                                    const SeqView& sv, const ltea_cache& cache, void* out, hipStream_t stream,
                                    float* lse = nullptr, const int32_t* kv_start = nullptr,
                                    const int32_t* kv_len = nullptr);
bool attention_mfma_supported(const ltea_cfg& cfg, int64_t kv_stride_tok, int32_t max_seqlen);
// sv packs the query / output rows.  With kv_start / kv_len (device, per sequence) the keys of sequence s are rows
// kv_start[s] .. +kv_len[s]-1 of k / v and its queries are the last positions of that key sequence; without
// them sv packs the keys too.
hipError_t launch_attention_mfma(const ltea_cfg& cfg, const void* q, int64_t q_stride_tok, int64_t q_stride_head,
                                 const void* k, const void* v, int64_t kv_stride_tok, int64_t kv_stride_head,
                                 const SeqView& sv, const ltea_cache& cache, void* out, hipStream_t stream,
                                 const int32_t* kv_start = nullptr, const int32_t* kv_len = nullptr,
                                 float* lse = nullptr);
// lse (optional, both launchers): [Hq][total_tokens] fp32, natural log of each query's softmax normaliser.

// ---- continuation of a prefill onto an existing cache ---------------------------------------------------
// Device buffers of the "extended sequences" (pad | old kept entries by position | ring tokens | new tokens) that
// the scoring, retention and attention launchers are then pointed at.
struct AppendBuffers {
  void* ext_k; void* ext_v;      // [total_ext][Hkv][D]
  void* ext_kf;                  // the keys the scoring kernels read: ext_k, or a buffer of its own (rotary models)
  float* ext_logits;             // [Hkv][total_ext]
  const int32_t* cu_ext;         // [n_seqs + 1]
  const int32_t* cu_score;       // [n_seqs + 1] packing handed to the scoring kernels (pad rows of sequences whose
                                 // ring begins at position 0 are left out of them)
  const int32_t* kv_start;       // first ring row of each sequence in the extended buffers
  const int32_t* kv_len;         // ring + new tokens of each sequence
  int32_t* local_pos;            // kept positions in the ring + new frame, [n_seqs][Hkv][budget]
  int64_t total_ext;             // row count the buffers are sized for (an upper bound of cu_ext[n_seqs])
  int32_t max_ext_len;           // upper bound of one extended sequence
};
int64_t append_ext_tokens(const ltea_cfg& cfg, int n_seqs, int64_t total_new);
size_t append_workspace(const ltea_cfg& cfg, int n_seqs, int64_t total_new, bool feature_keys);
hipError_t launch_append_build(const ltea_cfg& cfg, const void* k_new, const void* v_new, const void* kf_new,
                               int64_t stride_tok, int64_t stride_head, const int32_t* cu_new, int n_seqs,
                               int64_t total_new, int32_t max_new, const ltea_rope* rope, int32_t* status,
                               const ltea_cache& cache, void* workspace, AppendBuffers* out, hipStream_t stream);
hipError_t launch_append_keys(const ltea_cfg& cfg, int n_seqs, int64_t total_new, const ltea_cache& cache, int rho,
                              void* workspace, const AppendBuffers& buf, hipStream_t stream);
hipError_t launch_append_fixup(const ltea_cfg& cfg, const int32_t* cu_new, int n_seqs, int64_t total_new,
                               const ltea_cache& cache, int rho, void* workspace, hipStream_t stream);

// ---- (d) decode step -------------------------------------------------------------------------------
int decode_num_splits(const ltea_cfg& cfg, int n_seqs, bool scoring_inside);
size_t decode_workspace(const ltea_cfg& cfg, int n_seqs);                               // minimum
size_t decode_workspace_full(const ltea_cfg& cfg, const ltea_cnn& cnn, int n_seqs);     // enables every path
hipError_t launch_decode_step(const ltea_cfg& cfg, const ltea_cnn& cnn, const void* q, const void* k, const void* v,
                              void* out, const ltea_cache& cache, int n_seqs, void* workspace, size_t workspace_bytes,
                              hipStream_t stream);

// Eager step of a rotary model in three parts: the receptive-field windows of the tokens being finalised are packed
// (ring keys rotated back, the incoming key from k_feat or rotated back too), any prefill scoring launcher runs over
// them (2 * n_seqs pseudo-sequences `cu2`, rows of [Hkv][D]), and the step proper picks its logits from `logits`.
struct DecodeWindows {
  void* win_k; void* win_v;   // [n_seqs * (2 rho + 1)][Hkv][D]
  int32_t* cu2;               // [2 * n_seqs + 1]
  float* logits;              // [Hkv][total]
  int64_t total;              // n_seqs * (2 rho + 1)
};
size_t decode_windows_layout(const ltea_cfg& cfg, int rho, int n_seqs, void* base, DecodeWindows* out);
hipError_t launch_decode_windows(const ltea_cfg& cfg, int rho, const void* k, const void* v, const void* k_feat,
                                 const ltea_rope* rope, int32_t* status, const ltea_cache& cache, int n_seqs,
                                 const DecodeWindows& w, hipStream_t stream);
hipError_t launch_decode_step_scored(const ltea_cfg& cfg, const ltea_cnn& cnn, const void* q, const void* k,
                                     const void* v, void* out, const ltea_cache& cache, int n_seqs, void* workspace,
                                     const float* logits, int64_t logits_total, hipStream_t stream);

hipError_t launch_decode_step_lazy(const ltea_cfg& cfg, const void* q, const void* k, const void* v, void* out,
                                   const ltea_cache& cache, int n_seqs, int32_t* status, void* workspace,
                                   hipStream_t stream);

// ---- backward of the scoring CNN (cnn_backward.hip) ---------------------------------------------------------
size_t cnn_backward_workspace(const ltea_cfg& cfg, const ltea_cnn& cnn, int64_t total_tokens);
hipError_t launch_cnn_backward(const ltea_cfg& cfg, const ltea_cnn& cnn, const void* k, const void* v,
                               int64_t stride_tok, int64_t stride_head, const SeqView& sv, const float* dz,
                               const ltea_cnn_grad& grad, void* dk, void* dv, void* workspace, hipStream_t stream);

// ---- training-side backward --------------------------------------------------------------------------------
// kept: the compact arrays the retention launcher leaves when run with budget = kept_capacity and a cap that never
// binds (ascending kept out-of-window positions per (sequence, KV head) and their K / V rows).
// delta: [Hq][total] fp32 scratch; dq/dk/dv contiguous [total][H][D] of cfg.dtype; dz [Hkv][total]; counts [n_seqs][Hkv].
hipError_t launch_train_backward(const ltea_cfg& cfg, const void* q, int64_t q_st, int64_t q_sh, const void* k,
                                 const void* v, int64_t kv_st, int64_t kv_sh, const SeqView& sv, const void* out,
                                 const void* dout, const float* lse, const float* logits, const float* lambda,
                                 const ltea_cache& kept, int kept_capacity, float* delta, float* far_dk, float* far_dv,
                                 void* dq, void* dk, void* dv, float* dz, int32_t* counts, hipStream_t stream);
// far_dk / far_dv: fp32 scratch [train_far_chunks(n_seqs, Hkv)][n_seqs * Hkv][kept_capacity][D] each (used by the bf16 path).

// ---- deferred batched scoring of the decode cache ---------------------------------------------------------
struct RescoreBuffers {
  void* pk; void* pv;     // [n_seqs * window][Hkv][D] ring rows in position order (keys rotated back if asked)
  float* logits;          // [Hkv][n_seqs * window]
  int32_t* cu;            // [n_seqs + 1] = b * window
  int32_t* plan;          // [n_seqs][3] = first packed position, first newly final position, end of them
  int64_t total;          // n_seqs * window
};
// Carves the buffers from `base` (may be null when only the size is wanted); returns the bytes used.
size_t rescore_workspace(const ltea_cfg& cfg, int n_seqs, RescoreBuffers* out, void* base);
hipError_t launch_rescore_pack(const ltea_cfg& cfg, const ltea_rope* rope_or_null, const ltea_cache& cache, int n_seqs,
                               int rho, int32_t* status, const RescoreBuffers& buf, hipStream_t stream);
hipError_t launch_rescore_scatter(const ltea_cfg& cfg, const ltea_cache& cache, int n_seqs, const RescoreBuffers& buf,
                                  hipStream_t stream);

}  // namespace ltea
