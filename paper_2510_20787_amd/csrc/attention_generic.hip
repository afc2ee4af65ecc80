// Prefill attention over window + retained set (paper Section 3.1.3), generic fp32-VALU path.
//
// One wavefront per (query token, query head): keys are taken 64 at a time (one per lane) from the
// concatenation [window positions i-w+1..i] ++ [compact retained slots], retained entries still inside
// the query's window are masked, and an online softmax accumulates the output in fp32.  This path serves
// fp32 storage (and is the numerically plain reference shape of the computation); bf16 storage runs on
// the MFMA kernel instead.
#include "ltea_common.h"
#include "ltea_kernels.h"

namespace ltea {
namespace {

constexpr int kWavesPerBlock = 4;

template <typename T, int D>
__global__ void __launch_bounds__(kWavesPerBlock * kWave)
attention_generic_kernel(const T* __restrict__ q, int64_t q_st, int64_t q_sh, const T* __restrict__ k,
                         const T* __restrict__ v, int64_t kv_st, int64_t kv_sh, const int32_t* __restrict__ cu,
                         int n_seqs, int64_t total, int Hq, int Hkv, int window, int budget, float scale,
                         const T* __restrict__ k_ret, const T* __restrict__ v_ret,
                         const int32_t* __restrict__ ret_pos, const int32_t* __restrict__ ret_count,
                         T* __restrict__ out, float* __restrict__ lse, const int32_t* __restrict__ kv_start,
                         const int32_t* __restrict__ kv_len) {
  __shared__ float q_lds[kWavesPerBlock][D];
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const int64_t item = (int64_t)blockIdx.x * kWavesPerBlock + wave;
  const bool active = item < total * Hq;
  const int64_t tok = active ? item / Hq : 0;
  const int hq = active ? (int)(item - tok * Hq) : 0;
  const int h = hq / (Hq / Hkv);
  const int s = find_sequence(cu, n_seqs, tok);
  // cu packs the query / output rows.  Normally it packs the keys as well; with kv_start / kv_len given, the keys of
  // sequence s are rows kv_start[s] .. kv_start[s] + kv_len[s] - 1 of k / v and the queries are the last
  // cu[s+1] - cu[s] positions of that key sequence (continuation of a prefill).
  int64_t lo = cu[s];
  int i = (int)(tok - lo);
  if (kv_start != nullptr) {
    i += kv_len[s] - (int)(cu[s + 1] - lo);
    lo = kv_start[s];
  }
  const int wlo = i - window + 1 > 0 ? i - window + 1 : 0;
  const int n_win = i - wlo + 1;
  const int64_t head = (int64_t)s * Hkv + h;
  const int cnt = budget > 0 ? ret_count[head] : 0;
  const int n_items = n_win + cnt;

  const T* qr = q + tok * q_st + (int64_t)hq * q_sh;
  for (int m = lane; m < D; m += kWave) q_lds[wave][m] = to_f32(qr[m]);
  __syncthreads();
  if (!active) return;  // no barrier below this point

  float m_run = -INFINITY, l_run = 0.f;
  float acc[D / kWave];
#pragma unroll
  for (int e = 0; e < D / kWave; ++e) acc[e] = 0.f;

  for (int c0 = 0; c0 < n_items; c0 += kWave) {
    const int c = c0 + lane;
    bool valid = c < n_items;
    const T* kr = nullptr;
    if (valid) {
      if (c < n_win) {
        kr = k + (lo + wlo + c) * kv_st + (int64_t)h * kv_sh;
      } else {
        const int r = c - n_win;
        valid = ret_pos[head * budget + r] <= i - window;
        kr = k_ret + (head * budget + r) * D;
      }
    }
    float sc = -INFINITY;
    if (valid) {
      float dot = 0.f;
#pragma unroll 8
      for (int m = 0; m < D; ++m) dot = fmaf(q_lds[wave][m], to_f32(kr[m]), dot);
      sc = dot * scale;
    }
    const float m_new = fmaxf(m_run, wave_max(sc));
    if (m_new == -INFINITY) continue;  // nothing visible yet (uniform across the wave)
    const float p = valid ? expf(sc - m_new) : 0.f;
    const float alpha = expf(m_run - m_new);  // exp(-inf) = 0 on the first visible chunk
    l_run = l_run * alpha + wave_sum(p);
#pragma unroll
    for (int e = 0; e < D / kWave; ++e) acc[e] *= alpha;
    m_run = m_new;
    const int in_chunk = n_items - c0 < kWave ? n_items - c0 : kWave;
    for (int src = 0; src < in_chunk; ++src) {
      const float pj = __shfl(p, src, kWave);
      if (pj == 0.f) continue;  // uniform
      const int cs = c0 + src;
      const T* vr = cs < n_win ? v + (lo + wlo + cs) * kv_st + (int64_t)h * kv_sh
                               : v_ret + (head * budget + (cs - n_win)) * D;
#pragma unroll
      for (int e = 0; e < D / kWave; ++e) acc[e] = fmaf(pj, to_f32(vr[lane + e * kWave]), acc[e]);
    }
  }
  T* orow = out + (tok * Hq + hq) * D;
  const float inv = 1.0f / l_run;
#pragma unroll
  for (int e = 0; e < D / kWave; ++e) orow[lane + e * kWave] = from_f32<T>(acc[e] * inv);
  if (lse != nullptr && lane == 0) lse[(int64_t)hq * total + tok] = m_run + logf(l_run);  // wanted by a backward pass
}

template <typename T, int D>
hipError_t run(const ltea_cfg& cfg, const void* q, int64_t q_st, int64_t q_sh, const void* k, const void* v,
               int64_t kv_st, int64_t kv_sh, const SeqView& sv, const ltea_cache& c, void* out, float scale,
               float* lse, const int32_t* kv_start, const int32_t* kv_len, hipStream_t stream) {
  const int64_t items = sv.total_tokens * cfg.Hq;
  dim3 grid((unsigned)((items + kWavesPerBlock - 1) / kWavesPerBlock));
  hipLaunchKernelGGL((attention_generic_kernel<T, D>), grid, dim3(kWavesPerBlock * kWave), 0, stream,
                     static_cast<const T*>(q), q_st, q_sh, static_cast<const T*>(k), static_cast<const T*>(v), kv_st,
                     kv_sh, sv.cu_seqlens, sv.n_seqs, sv.total_tokens, cfg.Hq, cfg.Hkv, cfg.window, cfg.budget, scale,
                     static_cast<const T*>(c.k_ret), static_cast<const T*>(c.v_ret), c.ret_pos, c.ret_count,
                     static_cast<T*>(out), lse, kv_start, kv_len);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_attention_generic(const ltea_cfg& cfg, const void* q, int64_t q_st, int64_t q_sh, const void* k,
                                    const void* v, int64_t kv_st, int64_t kv_sh, const SeqView& sv,
                                    const ltea_cache& c, void* out, hipStream_t stream, float* lse,
                                    const int32_t* kv_start, const int32_t* kv_len) {
  if (sv.total_tokens == 0) return hipSuccess;
  const float scale = cfg.softmax_scale > 0.f ? cfg.softmax_scale : 1.0f / sqrtf((float)cfg.D);
  if (cfg.dtype == LTEA_F32) {
    return cfg.D == 64 ? run<float, 64>(cfg, q, q_st, q_sh, k, v, kv_st, kv_sh, sv, c, out, scale, lse, kv_start, kv_len, stream)
                       : run<float, 128>(cfg, q, q_st, q_sh, k, v, kv_st, kv_sh, sv, c, out, scale, lse, kv_start, kv_len, stream);
  }
  return cfg.D == 64 ? run<bf16_t, 64>(cfg, q, q_st, q_sh, k, v, kv_st, kv_sh, sv, c, out, scale, lse, kv_start, kv_len, stream)
                     : run<bf16_t, 128>(cfg, q, q_st, q_sh, k, v, kv_st, kv_sh, sv, c, out, scale, lse, kv_start, kv_len, stream);
}

}  // namespace ltea
