// Scoring CNN of the LTE module (paper Section 3.1.1; Appendix A), generic layered path.
//
// Any depth, fp32 or bf16 storage, plain fp32 VALU arithmetic: one launch per conv layer (activations
// of layer l go through a [Hkv][T][C_l] fp32 scratch array) plus one launch for the per-head output
// projection.  It is the path for fp32 inputs and for multi-layer stacks; the single-layer bf16 case has
// a fused MFMA kernel of its own.
#include "ltea_common.h"
#include "ltea_kernels.h"

namespace ltea {
namespace {

// One thread per (token, output channel) of one KV head.
// first != 0: input features are concat(K row, V row) of the token (2*D channels, keys first).
// first == 0: input is act_in [Hkv][T][Cin] fp32.
// Tap t reads position j + (t - (ks-1)/2) * dil of the same sequence; outside -> 0 (zero padding at
// every layer).  Output = Swish(bias + sum).
template <typename T>
__global__ void __launch_bounds__(256)
conv_layer_kernel(const T* __restrict__ k, const T* __restrict__ v, int64_t stride_tok, int64_t stride_head, int D,
                  const float* __restrict__ act_in, int first, const T* __restrict__ W,
                  const float* __restrict__ bias, int Cin, int Cout, int ks, int dil,
                  const int32_t* __restrict__ cu, int n_seqs, int64_t total, float* __restrict__ act_out) {
  const int h = blockIdx.y;
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t tok = idx / Cout;
  const int c = (int)(idx - tok * Cout);
  if (tok >= total) return;
  const int s = find_sequence(cu, n_seqs, tok);
  const int64_t lo = cu[s], hi = cu[s + 1];
  const T* Wc = W + ((int64_t)h * Cout + c) * Cin * ks;
  float acc = bias[(int64_t)h * Cout + c];
  const int half = (ks - 1) / 2;
  for (int t = 0; t < ks; ++t) {
    const int64_t p = tok + (int64_t)(t - half) * dil;
    if (p < lo || p >= hi) continue;
    if (first) {
      const T* kr = k + p * stride_tok + (int64_t)h * stride_head;
      const T* vr = v + p * stride_tok + (int64_t)h * stride_head;
      for (int m = 0; m < D; ++m) acc = fmaf(to_f32(kr[m]), to_f32(Wc[(int64_t)m * ks + t]), acc);
      for (int m = 0; m < D; ++m) acc = fmaf(to_f32(vr[m]), to_f32(Wc[(int64_t)(D + m) * ks + t]), acc);
    } else {
      const float* ar = act_in + ((int64_t)h * total + p) * Cin;
      for (int m = 0; m < Cin; ++m) acc = fmaf(ar[m], to_f32(Wc[(int64_t)m * ks + t]), acc);
    }
  }
  act_out[((int64_t)h * total + tok) * Cout + c] = silu_f32(acc);
}

// logits[h][t] = b_out[h] + sum_c w_out[h][c] * act[h][t][c]
template <typename T>
__global__ void __launch_bounds__(256)
out_proj_kernel(const float* __restrict__ act, const T* __restrict__ w_out, const float* __restrict__ b_out, int C,
                int64_t total, float* __restrict__ logits) {
  const int h = blockIdx.y;
  const int64_t tok = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (tok >= total) return;
  const float* a = act + ((int64_t)h * total + tok) * C;
  float acc = b_out[h];
  for (int c = 0; c < C; ++c) acc = fmaf(a[c], to_f32(w_out[(int64_t)h * C + c]), acc);
  logits[(int64_t)h * total + tok] = acc;
}

template <typename T>
hipError_t run(const ltea_cfg& cfg, const ltea_cnn& cnn, const void* k, const void* v, int64_t stride_tok,
               int64_t stride_head, const SeqView& sv, float* logits, void* workspace, hipStream_t stream) {
  const int64_t total = sv.total_tokens;
  int cmax = 0;
  for (int l = 0; l < cnn.n_layers; ++l) cmax = cnn.c_out[l] > cmax ? cnn.c_out[l] : cmax;
  float* buf[2] = {static_cast<float*>(workspace), static_cast<float*>(workspace) + (int64_t)cfg.Hkv * total * cmax};
  int cin = 2 * cfg.D;
  const float* act_in = nullptr;
  for (int l = 0; l < cnn.n_layers; ++l) {
    const int cout = cnn.c_out[l];
    float* act_out = buf[l & 1];
    const int64_t work = total * cout;
    dim3 grid((unsigned)((work + 255) / 256), (unsigned)cfg.Hkv);
    hipLaunchKernelGGL(conv_layer_kernel<T>, grid, dim3(256), 0, stream, static_cast<const T*>(k),
                       static_cast<const T*>(v), stride_tok, stride_head, cfg.D, act_in, l == 0 ? 1 : 0,
                       static_cast<const T*>(cnn.w[l]), cnn.bias[l], cin, cout, cnn.kernel[l], cnn.dilation[l],
                       sv.cu_seqlens, sv.n_seqs, total, act_out);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    act_in = act_out;
    cin = cout;
  }
  dim3 grid((unsigned)((total + 255) / 256), (unsigned)cfg.Hkv);
  hipLaunchKernelGGL(out_proj_kernel<T>, grid, dim3(256), 0, stream, act_in, static_cast<const T*>(cnn.w_out),
                     cnn.b_out, cin, total, logits);
  return hipGetLastError();
}

}  // namespace

size_t score_generic_workspace(const ltea_cfg& cfg, const ltea_cnn& cnn, int64_t total_tokens) {
  int cmax = 0;
  for (int l = 0; l < cnn.n_layers; ++l) cmax = cnn.c_out[l] > cmax ? cnn.c_out[l] : cmax;
  const size_t one = (size_t)cfg.Hkv * (size_t)total_tokens * (size_t)cmax * sizeof(float);
  return cnn.n_layers > 1 ? 2 * one : one;
}

hipError_t launch_score_generic(const ltea_cfg& cfg, const ltea_cnn& cnn, const void* k, const void* v,
                                int64_t stride_tok, int64_t stride_head, const SeqView& sv, float* logits,
                                void* workspace, hipStream_t stream) {
  if (sv.total_tokens == 0) return hipSuccess;
  if (cfg.dtype == LTEA_F32)
    return run<float>(cfg, cnn, k, v, stride_tok, stride_head, sv, logits, workspace, stream);
  return run<bf16_t>(cfg, cnn, k, v, stride_tok, stride_head, sv, logits, workspace, stream);
}

}  // namespace ltea
