// Arguments shared by the training-side backward kernels (generic and matrix-core paths).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ltea {

constexpr int kTrainFarChunksMax = 8;
// Shares of the query range in the far pass of dK / dV (= scratch slices): enough of them that a small batch still
// yields a few hundred workgroups of similar length, a single one when there are plenty of (sequence, head) pairs.
inline int train_far_chunks(int n_seqs, int Hkv) {
  const long heads = (long)n_seqs * Hkv;
  long c = heads > 0 ? (256 + heads - 1) / heads : 1;
  return (int)(c < 1 ? 1 : (c > kTrainFarChunksMax ? kTrainFarChunksMax : c));
}

struct TrainArgs {
  const void *q, *k, *v, *out, *dout;
  int64_t q_st, q_sh, kv_st, kv_sh;
  const int32_t* cu;
  int n_seqs;
  int64_t total;
  int Hq, Hkv, window, budget, sink;
  float scale, tau;
  const int32_t *ret_pos, *ret_count;   // compacted candidates of the forward: ascending positions, row pitch `budget`
  const void *k_ret, *v_ret;            // their K / V rows, [n_seqs][Hkv][budget][D]
  int max_seqlen;
  int far_chunks;                       // train_far_chunks(n_seqs, Hkv)
  const float *lse, *logits, *lambda;
  float* delta;
  float *far_dk, *far_dv;               // fp32 scratch of the matrix-core dK / dV path, far_chunks slices laid out like k_ret / v_ret
  void *dq, *dk, *dv;
  float* dz;
  int32_t* counts;
};

// bf16 path on MFMA (train_mfma.hip).
bool train_mfma_supported(const TrainArgs& A, int D);
hipError_t launch_train_backward_mfma(const TrainArgs& A, int D, hipStream_t stream);

}  // namespace ltea
