// Scoring CNN of the LTE module (paper Section 3.1.1; Appendix A): fused single-layer bf16 path on MFMA.
//
//   z[h][j] = b_out[h] + sum_c w_out[h][c] * Swish( bias[h][c] + sum_{t,m} W[h][c][m][t] * x[j + (t-half)*dil][m] )
// with x = concat(key, value) of the token (2*D channels).  The contraction over (tap, channel) is a small
// GEMM per head: out^T[c, token] = W_t[c, :] . X^T[:, token + shift_t], run on v_mfma_f32_32x32x16_bf16 with
// the (zero-padded to 32) channels as MFMA rows and 32 tokens per wave as MFMA columns.  In the accumulator
// layout one lane owns one token, so bias, Swish and the output projection are per-lane work on the 16
// channel values it holds plus one exchange with the lane holding the other 16.
//
// One workgroup = 128 consecutive tokens of one (sequence, KV head).  The token tile with its halo of
// half*dil rows on each side (zeros outside the sequence) is staged once in LDS, K and V rows coalesced in
// 16-byte pieces; the weights of one tap at a time are staged in a double-buffered LDS panel while the
// previous tap is being multiplied.
#include "ltea_common.h"
#include "ltea_kernels.h"

namespace ltea {
namespace {

constexpr int TM = 128;       // tokens per workgroup
constexpr int kThreads = 256;
constexpr int CP = 32;        // channels padded to one MFMA tile

template <int D>
__global__ void __launch_bounds__(kThreads)
score_mfma_kernel(const bf16_t* __restrict__ k, const bf16_t* __restrict__ v, int64_t st, int64_t sh,
                  const bf16_t* __restrict__ W, const float* __restrict__ bias, const bf16_t* __restrict__ w_out,
                  const float* __restrict__ b_out, int C, int ks, int dil, const int32_t* __restrict__ cu,
                  int n_seqs, int tiles_upper, int64_t total, float* __restrict__ logits) {
  constexpr int C2 = 2 * D;        // input channels
  constexpr int XS = C2 + 8;       // LDS row stride (elements) of the token tile and of the weight panel
  constexpr int PPR = C2 / 8;      // 16-byte pieces per token row
  constexpr int RPP = kThreads / PPR;
  constexpr int WPT = C2 * CP / kThreads;  // weight elements per thread per tap
  extern __shared__ __align__(16) unsigned char smem[];
  const int half = (ks - 1) / 2, rho = half * dil;
  const int rows = TM + 2 * rho;
  bf16_t* x_lds = reinterpret_cast<bf16_t*>(smem);
  bf16_t* w_lds = x_lds + (size_t)rows * XS;  // two panels of CP x XS

  const int h = blockIdx.y;
  int tile = blockIdx.x, s = 0, n = 0;
  for (; s < n_seqs; ++s) {
    n = cu[s + 1] - cu[s];
    const int nt = (n + TM - 1) / TM;
    if (tile < nt) break;
    tile -= nt;
  }
  if (s == n_seqs) return;
  const int64_t lo = cu[s];
  const int j0 = tile * TM;
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, ql = lane & 31, hb = lane >> 5;

  // ---- token tile with halo -> LDS -----------------------------------------------------------------------
  {
    const int piece = tid % PPR, r_in = tid / PPR;
    const bool is_v = piece >= PPR / 2;
    const bf16_t* base = (is_v ? v : k) + (int64_t)h * sh + (is_v ? piece - PPR / 2 : piece) * 8;
    for (int r = r_in; r < rows; r += RPP) {
      const int p = j0 - rho + r;
      u32x4 x = {0u, 0u, 0u, 0u};
      if (p >= 0 && p < n) x = *reinterpret_cast<const u32x4*>(base + (lo + p) * st);
      *reinterpret_cast<u32x4*>(&x_lds[r * XS + piece * 8]) = x;
    }
  }
  // ---- weight panel of one tap: w_panel[c][m] = W[h][c][m][tap] (zero rows for c >= C) -----------------------
  const bf16_t* Wh = W + (int64_t)h * C * C2 * ks;
  uint16_t wreg[WPT];
  auto load_panel = [&](int tap) {
#pragma unroll
    for (int i = 0; i < WPT; ++i) {
      const int e = tid + kThreads * i;
      const int c = e / C2, m = e - c * C2;
      wreg[i] = c < C ? reinterpret_cast<const uint16_t*>(Wh)[((int64_t)c * C2 + m) * ks + tap] : (uint16_t)0;
    }
  };
  auto store_panel = [&](int buf) {
    uint16_t* dst = reinterpret_cast<uint16_t*>(w_lds + (size_t)buf * CP * XS);
#pragma unroll
    for (int i = 0; i < WPT; ++i) {
      const int e = tid + kThreads * i;
      const int c = e / C2, m = e - c * C2;
      dst[c * XS + m] = wreg[i];
    }
  };
  load_panel(0);
  store_panel(0);
  __syncthreads();

  f32x16 acc;
#pragma unroll
  for (int r = 0; r < 16; ++r) acc[r] = 0.f;
  for (int tap = 0; tap < ks; ++tap) {
    if (tap + 1 < ks) load_panel(tap + 1);
    const bf16_t* a_row = w_lds + (size_t)(tap & 1) * CP * XS + ql * XS + 8 * hb;          // channel ql
    const bf16_t* b_row = x_lds + (size_t)(32 * wv + ql + tap * dil) * XS + 8 * hb;        // token 32*wv+ql, shifted
#pragma unroll
    for (int mc = 0; mc < C2 / 16; ++mc) {
      const bf16x8 a = *reinterpret_cast<const bf16x8*>(a_row + 16 * mc);
      const bf16x8 b = *reinterpret_cast<const bf16x8*>(b_row + 16 * mc);
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc, 0, 0, 0);
    }
    if (tap + 1 < ks) store_panel((tap + 1) & 1);
    __syncthreads();
  }

  // ---- epilogue: accumulator register r of lane half hb is channel 8*(r/4) + 4*hb + r%4 of token ql ----------
  float z = 0.f;
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    const int c = 8 * (r / 4) + 4 * hb + (r % 4);
    if (c < C) {
      const float y = acc[r] + bias[h * C + c];
      const float a = y * __frcp_rn(1.0f + __expf(-y));
      z = fmaf(a, to_f32(w_out[h * C + c]), z);
    }
  }
  z += __shfl_xor(z, 32, kWave);
  const int j = j0 + 32 * wv + ql;
  if (hb == 0 && j < n) logits[(int64_t)h * total + lo + j] = z + b_out[h];
}

size_t lds_bytes(int D, int ks, int dil) {
  const int rho = (ks - 1) / 2 * dil;
  return ((size_t)(TM + 2 * rho) + 2 * CP) * (2 * D + 8) * sizeof(uint16_t);
}

template <int D>
hipError_t run(const ltea_cfg& cfg, const ltea_cnn& cnn, const void* k, const void* v, int64_t st, int64_t sh,
               const SeqView& sv, float* logits, hipStream_t stream) {
  const size_t lds = lds_bytes(D, cnn.kernel[0], cnn.dilation[0]);
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&score_mfma_kernel<D>),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  if (e != hipSuccess) return e;
  const int64_t tiles_upper = (sv.total_tokens + TM - 1) / TM + sv.n_seqs;
  hipLaunchKernelGGL(score_mfma_kernel<D>, dim3((unsigned)tiles_upper, (unsigned)cfg.Hkv), dim3(kThreads), lds, stream,
                     static_cast<const bf16_t*>(k), static_cast<const bf16_t*>(v), st, sh,
                     static_cast<const bf16_t*>(cnn.w[0]), cnn.bias[0], static_cast<const bf16_t*>(cnn.w_out),
                     cnn.b_out, cnn.c_out[0], cnn.kernel[0], cnn.dilation[0], sv.cu_seqlens, sv.n_seqs,
                     (int)tiles_upper, sv.total_tokens, logits);
  return hipGetLastError();
}

}  // namespace

bool score_mfma_supported(const ltea_cfg& cfg, const ltea_cnn& cnn) {
  if (cfg.dtype != LTEA_BF16 || cnn.n_layers != 1 || cnn.c_out[0] > CP) return false;
  if (cfg.D != 64 && cfg.D != 128) return false;
  return lds_bytes(cfg.D, cnn.kernel[0], cnn.dilation[0]) <= 150 * 1024;
}

hipError_t launch_score_mfma(const ltea_cfg& cfg, const ltea_cnn& cnn, const void* k, const void* v, int64_t st,
                             int64_t sh, const SeqView& sv, float* logits, hipStream_t stream) {
  if (sv.total_tokens == 0) return hipSuccess;
  return cfg.D == 64 ? run<64>(cfg, cnn, k, v, st, sh, sv, logits, stream)
                     : run<128>(cfg, cnn, k, v, st, sh, sv, logits, stream);
}

}  // namespace ltea
