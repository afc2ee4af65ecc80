// Training-side backward of the SWA+LTE attention (paper Section 3.1.2 "Adaptive training"; Algorithm 1).
//
// The forward of training is the prefill pipeline with the budget lifted (uncapped eq. 5): scoring, compaction of
// every candidate, window + kept attention, plus the softmax normaliser of every query.  This file holds what the
// backward adds:
//
//   train_dq_kernel   one wave per (query, query head): delta = <dO, O>, then over the keys the query saw (its
//                     window and the kept positions that had left it) p = exp(scale q.k - lse),
//                     dS = p (dO.v - delta) scale, dQ = sum dS k.  Writes dQ and delta.
//   train_dkv_kernel  one wave per (key, KV head): over the (query, query head of the group) pairs that saw the
//                     key (queries j .. j+w-1, and all later ones if the key is a candidate) the same p and dS,
//                     dV = sum p dO, dK = sum dS q; then the surrogate gradient of the retention score
//                     d r_j := <v_j, dV_j> (straight-through estimator), the sparsity penalty's lambda_h 1[r_j > r_tau],
//                     both through the sigmoid's slope into d z_j; and the per-(sequence, head) retention counts.
//
// Both kernels give one lane one key (or one query) for the two dot products, then broadcast the lane results
// and let the lanes own the feature dimension for the rank-1 updates: fp32 VALU arithmetic, every row read as
// whole 128/256-byte rows.  Results do not depend on launch order (no floating-point atomics).
#include <type_traits>

#include "ltea_common.h"
#include "ltea_kernels.h"
#include "train_common.h"

namespace ltea {
namespace {

constexpr int kWavesPerBlock = 4;


template <typename T, int D>
__global__ void __launch_bounds__(kWavesPerBlock * kWave)
train_dq_kernel(TrainArgs A) {
  constexpr int EPL = D / kWave;   // features per lane when the lanes own the feature dimension
  __shared__ float q_lds[kWavesPerBlock][D], do_lds[kWavesPerBlock][D];
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const int64_t item = (int64_t)blockIdx.x * kWavesPerBlock + wave;
  const bool active = item < A.total * A.Hq;
  const int64_t tok = active ? item / A.Hq : 0;
  const int hq = active ? (int)(item - tok * A.Hq) : 0;
  const int h = hq / (A.Hq / A.Hkv);
  const int s = find_sequence(A.cu, A.n_seqs, tok);
  const int64_t lo = A.cu[s];
  const int i = (int)(tok - lo);
  const T* q = static_cast<const T*>(A.q);
  const T* k = static_cast<const T*>(A.k);
  const T* v = static_cast<const T*>(A.v);
  const T* qr = q + tok * A.q_st + (int64_t)hq * A.q_sh;
  const T* orow = static_cast<const T*>(A.out) + (tok * A.Hq + hq) * D;
  const T* dorow = static_cast<const T*>(A.dout) + (tok * A.Hq + hq) * D;
  float dsum = 0.f;
#pragma unroll
  for (int e = 0; e < EPL; ++e) {
    const int m = lane + e * kWave;
    const float d_o = to_f32(dorow[m]);
    q_lds[wave][m] = to_f32(qr[m]);
    do_lds[wave][m] = d_o;
    dsum = fmaf(d_o, to_f32(orow[m]), dsum);
  }
  const float delta = wave_sum(dsum);
  __syncthreads();
  if (!active) return;  // no barrier below this point
  if (lane == 0) A.delta[(int64_t)hq * A.total + tok] = delta;
  const float lse = A.lse[(int64_t)hq * A.total + tok];

  const int wlo = i - A.window + 1 > 0 ? i - A.window + 1 : 0;
  const int n_win = i - wlo + 1;
  const int64_t head = (int64_t)s * A.Hkv + h;
  const int32_t* rp = A.ret_pos + head * A.budget;
  // kept positions are ascending: the ones that have left this query's window are a prefix of the list
  int n_far = 0;
  {
    int a = 0, b = A.budget > 0 ? A.ret_count[head] : 0;   // first index with rp[idx] > i - window, in [a, b]
    while (a < b) {
      const int mid = (a + b) >> 1;
      if (rp[mid] <= i - A.window) a = mid + 1; else b = mid;
    }
    n_far = a;
  }
  const int n_items = n_win + n_far;
  float acc[EPL];
#pragma unroll
  for (int e = 0; e < EPL; ++e) acc[e] = 0.f;
  for (int c0 = 0; c0 < n_items; c0 += kWave) {
    const int c = c0 + lane;
    float ds = 0.f;
    if (c < n_items) {
      const int j = c < n_win ? wlo + c : rp[c - n_win];
      const T* kr = k + (lo + j) * A.kv_st + (int64_t)h * A.kv_sh;
      const T* vr = v + (lo + j) * A.kv_st + (int64_t)h * A.kv_sh;
      float dot = 0.f, dpv = 0.f;
#pragma unroll 8
      for (int m = 0; m < D; ++m) {
        dot = fmaf(q_lds[wave][m], to_f32(kr[m]), dot);
        dpv = fmaf(do_lds[wave][m], to_f32(vr[m]), dpv);
      }
      const float p = expf(fmaf(dot, A.scale, -lse));
      ds = p * (dpv - delta) * A.scale;
    }
    const int in_chunk = n_items - c0 < kWave ? n_items - c0 : kWave;
    for (int src = 0; src < in_chunk; ++src) {
      const float dsj = __shfl(ds, src, kWave);
      const int cs = c0 + src;
      const int j = cs < n_win ? wlo + cs : rp[cs - n_win];
      const T* kr = k + (lo + j) * A.kv_st + (int64_t)h * A.kv_sh;
#pragma unroll
      for (int e = 0; e < EPL; ++e) acc[e] = fmaf(dsj, to_f32(kr[lane + e * kWave]), acc[e]);
    }
  }
  T* dqr = static_cast<T*>(A.dq) + (tok * A.Hq + hq) * D;
#pragma unroll
  for (int e = 0; e < EPL; ++e) dqr[lane + e * kWave] = from_f32<T>(acc[e]);
}

template <typename T, int D>
__global__ void __launch_bounds__(kWavesPerBlock * kWave)
train_dkv_kernel(TrainArgs A) {
  constexpr int EPL = D / kWave;
  __shared__ float k_lds[kWavesPerBlock][D], v_lds[kWavesPerBlock][D];
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const int64_t item = (int64_t)blockIdx.x * kWavesPerBlock + wave;
  const bool active = item < A.total * A.Hkv;
  const int64_t tok = active ? item / A.Hkv : 0;
  const int h = active ? (int)(item - tok * A.Hkv) : 0;
  const int G = A.Hq / A.Hkv;
  const int s = find_sequence(A.cu, A.n_seqs, tok);
  const int64_t lo = A.cu[s];
  const int n = A.cu[s + 1] - (int)lo;
  const int j = (int)(tok - lo);
  const T* q = static_cast<const T*>(A.q);
  const T* dout = static_cast<const T*>(A.dout);
  const T* kr = static_cast<const T*>(A.k) + tok * A.kv_st + (int64_t)h * A.kv_sh;
  const T* vr = static_cast<const T*>(A.v) + tok * A.kv_st + (int64_t)h * A.kv_sh;
#pragma unroll
  for (int e = 0; e < EPL; ++e) {
    k_lds[wave][lane + e * kWave] = to_f32(kr[lane + e * kWave]);
    v_lds[wave][lane + e * kWave] = to_f32(vr[lane + e * kWave]);
  }
  __syncthreads();
  if (!active) return;  // no barrier below this point
  const float z = A.logits[(int64_t)h * A.total + tok];
  const bool above = z > A.tau;                       // NaN never passes
  const bool kept = j < A.sink || above;
  const int end = kept ? n : (j + A.window < n ? j + A.window : n);   // queries j .. end-1 saw this key
  const int n_items = (end - j) * G;
  float accv[EPL], acck[EPL];
#pragma unroll
  for (int e = 0; e < EPL; ++e) { accv[e] = 0.f; acck[e] = 0.f; }
  for (int c0 = 0; c0 < n_items; c0 += kWave) {
    const int c = c0 + lane;
    float p = 0.f, ds = 0.f;
    if (c < n_items) {
      const int i = j + c / G, hq = h * G + c % G;
      const T* qr = q + (lo + i) * A.q_st + (int64_t)hq * A.q_sh;
      const T* dor = dout + ((lo + i) * A.Hq + hq) * D;
      float dot = 0.f, dpv = 0.f;
#pragma unroll 8
      for (int m = 0; m < D; ++m) {
        dot = fmaf(k_lds[wave][m], to_f32(qr[m]), dot);
        dpv = fmaf(v_lds[wave][m], to_f32(dor[m]), dpv);
      }
      const int64_t qi = (int64_t)hq * A.total + lo + i;
      p = expf(fmaf(dot, A.scale, -A.lse[qi]));
      ds = p * (dpv - A.delta[qi]) * A.scale;
    }
    const int in_chunk = n_items - c0 < kWave ? n_items - c0 : kWave;
    for (int src = 0; src < in_chunk; ++src) {
      const float pj = __shfl(p, src, kWave), dsj = __shfl(ds, src, kWave);
      const int cs = c0 + src;
      const int i = j + cs / G, hq = h * G + cs % G;
      const T* qr = q + (lo + i) * A.q_st + (int64_t)hq * A.q_sh;
      const T* dor = dout + ((lo + i) * A.Hq + hq) * D;
#pragma unroll
      for (int e = 0; e < EPL; ++e) {
        accv[e] = fmaf(pj, to_f32(dor[lane + e * kWave]), accv[e]);
        acck[e] = fmaf(dsj, to_f32(qr[lane + e * kWave]), acck[e]);
      }
    }
  }
  T* dkr = static_cast<T*>(A.dk) + (tok * A.Hkv + h) * D;
  T* dvr = static_cast<T*>(A.dv) + (tok * A.Hkv + h) * D;
  float ste = 0.f;
#pragma unroll
  for (int e = 0; e < EPL; ++e) {
    dkr[lane + e * kWave] = from_f32<T>(acck[e]);
    dvr[lane + e * kWave] = from_f32<T>(accv[e]);
    ste = fmaf(accv[e], v_lds[wave][lane + e * kWave], ste);
  }
  ste = wave_sum(ste);
  if (lane == 0) {
    const float r = 1.0f / (1.0f + expf(-z));
    A.dz[(int64_t)h * A.total + tok] = (ste + (above ? A.lambda[h] : 0.f)) * r * (1.0f - r);
    if (above) atomicAdd(&A.counts[s * A.Hkv + h], 1);   // integer: the result does not depend on the order
  }
}

__global__ void __launch_bounds__(256) train_zero_counts_kernel(int32_t* counts, int n) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < n) counts[i] = 0;
}

template <typename T, int D>
hipError_t run(const TrainArgs& A, hipStream_t stream) {
  const int n_counts = A.n_seqs * A.Hkv;
  hipLaunchKernelGGL(train_zero_counts_kernel, dim3((unsigned)((n_counts + 255) / 256)), dim3(256), 0, stream, A.counts,
                     n_counts);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (A.total == 0) return hipSuccess;
  const int64_t qi = A.total * A.Hq, ki = A.total * A.Hkv;
  const dim3 qgrid((unsigned)((qi + kWavesPerBlock - 1) / kWavesPerBlock)), block(kWavesPerBlock * kWave);
  if constexpr (std::is_same<T, bf16_t>::value) {
    if (train_mfma_supported(A, D)) {
      return launch_train_backward_mfma(A, D, stream);   // matrix-core path
    }
  }
  hipLaunchKernelGGL((train_dq_kernel<T, D>), qgrid, block, 0, stream, A);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((train_dkv_kernel<T, D>), dim3((unsigned)((ki + kWavesPerBlock - 1) / kWavesPerBlock)), block, 0,
                     stream, A);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_train_backward(const ltea_cfg& cfg, const void* q, int64_t q_st, int64_t q_sh, const void* k,
                                 const void* v, int64_t kv_st, int64_t kv_sh, const SeqView& sv, const void* out,
                                 const void* dout, const float* lse, const float* logits, const float* lambda,
                                 const ltea_cache& kept, int kept_capacity, float* delta, float* far_dk, float* far_dv,
                                 void* dq, void* dk, void* dv, float* dz, int32_t* counts, hipStream_t stream) {
  if (sv.n_seqs == 0) return hipSuccess;
  TrainArgs A;
  A.q = q; A.k = k; A.v = v; A.out = out; A.dout = dout;
  A.q_st = q_st; A.q_sh = q_sh; A.kv_st = kv_st; A.kv_sh = kv_sh;
  A.cu = sv.cu_seqlens; A.n_seqs = sv.n_seqs; A.total = sv.total_tokens;
  A.Hq = cfg.Hq; A.Hkv = cfg.Hkv; A.window = cfg.window; A.budget = kept_capacity; A.sink = cfg.sink;
  A.scale = cfg.softmax_scale > 0.f ? cfg.softmax_scale : 1.0f / sqrtf((float)cfg.D);
  A.tau = cfg.tau_logit;
  A.ret_pos = kept.ret_pos; A.ret_count = kept.ret_count; A.k_ret = kept.k_ret; A.v_ret = kept.v_ret;
  A.max_seqlen = sv.max_seqlen;
  A.far_chunks = train_far_chunks(sv.n_seqs, cfg.Hkv);
  A.lse = lse; A.logits = logits; A.lambda = lambda; A.delta = delta; A.far_dk = far_dk; A.far_dv = far_dv;
  A.dq = dq; A.dk = dk; A.dv = dv; A.dz = dz; A.counts = counts;
  if (cfg.dtype == LTEA_F32) return cfg.D == 64 ? run<float, 64>(A, stream) : run<float, 128>(A, stream);
  return cfg.D == 64 ? run<bf16_t, 64>(A, stream) : run<bf16_t, 128>(A, stream);
}

}  // namespace ltea
