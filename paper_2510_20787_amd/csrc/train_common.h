// Arguments shared by the training-side backward kernels (generic and matrix-core paths).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ltea {

constexpr int kTrainFarChunks = 8;   // shares of the query range in the far pass of dK / dV (= scratch slices)

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
  const float *lse, *logits, *lambda;
  float* delta;
  float *far_dk, *far_dv;               // fp32 scratch of the matrix-core dK / dV path, kTrainFarChunks slices laid out like k_ret / v_ret
  void *dq, *dk, *dv;
  float* dz;
  int32_t* counts;
};

// bf16 path on MFMA (train_mfma.hip).
bool train_mfma_supported(const TrainArgs& A, int D);
hipError_t launch_train_backward_mfma(const TrainArgs& A, int D, hipStream_t stream);

}  // namespace ltea
