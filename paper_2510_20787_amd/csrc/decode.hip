// One decode step of the SWA+LTE cache (paper Section 3.1.3: cache replacement, decode attention and
// the deferred scoring of Section 3.1.1 item 2).
//
// Three launches per step, all on the caller's stream:
//   decode_update_kernel   one workgroup per (sequence, KV head): finalises the logit of position t-rho
//                          from the 2*rho newest ring rows plus the incoming token (any CNN depth, the
//                          activation pyramid lives in LDS), pops position t-window from the ring and
//                          inserts it into / lets it displace the worst entry of the compact segment,
//                          then writes k_t, v_t into ring slot t % window.
//   decode_attention_kernel  the memory-bound part: grid (sequence x KV head, split); every split streams
//                          its share of the [ring rows ++ compact rows] with 16-byte loads, one row per
//                          group of D*sizeof(T)/16 lanes, several rows in flight per lane, and keeps an
//                          online-softmax partial (max, sum, D accumulators) per query head.
//   decode_combine_kernel  merges the split partials, writes the output row and advances n_seen/n_scored.
#include "ltea_common.h"
#include "ltea_kernels.h"

namespace ltea {
namespace {

constexpr int kUpdThreads = 256;
constexpr int kConvSplit = 8;    // lanes cooperating on one conv output in the update kernel
constexpr int kAttnThreads = 256;
constexpr int kRowsInFlight = 4;  // rows per lane group per iteration of the streaming loop

// --------------------------------------------------------------------------------------------------
// update: scoring of t-rho, eviction of t-window, append of t
// --------------------------------------------------------------------------------------------------
struct CnnDev {
  int n_layers;
  int kernel[LTEA_MAX_CNN_LAYERS], dilation[LTEA_MAX_CNN_LAYERS], c_out[LTEA_MAX_CNN_LAYERS];
  const void* w[LTEA_MAX_CNN_LAYERS];
  const float* bias[LTEA_MAX_CNN_LAYERS];
  const void* w_out;
  const float* b_out;
};

template <typename T>
__global__ void __launch_bounds__(kUpdThreads)
decode_update_kernel(CnnDev cnn, int rho, int lds_row_floats, const T* __restrict__ k_new,
                     const T* __restrict__ v_new, int Hkv, int D, int window, int budget, int sink, float tau,
                     T* __restrict__ k_win, T* __restrict__ v_win, float* __restrict__ win_score,
                     T* __restrict__ k_ret, T* __restrict__ v_ret, float* __restrict__ ret_score,
                     int32_t* __restrict__ ret_pos, int32_t* __restrict__ ret_count,
                     const int32_t* __restrict__ n_seen) {
  extern __shared__ float lds[];  // two activation buffers of (2*rho+1) rows x lds_row_floats
  __shared__ unsigned long long red[kUpdThreads / kWave];
  __shared__ int worst_slot;
  const int tid = threadIdx.x;
  const int b = blockIdx.x / Hkv, h = blockIdx.x - b * Hkv;
  const int64_t head = (int64_t)b * Hkv + h;
  const int t = n_seen[b];
  const int slot = t % window;
  const int rows0 = 2 * rho + 1;
  float* buf_a = lds;
  float* buf_b = lds + (size_t)rows0 * lds_row_floats;

  // logit of the token that leaves the window; read before anything is written this step
  const int e_pos = t - window;
  const float z_e = e_pos >= 0 ? win_score[head * window + slot] : 0.f;
  const int cnt = ret_count[head];

  // ---- 1. final logit of position j = t - rho --------------------------------------------------
  const int j_fin = t - rho;
  if (j_fin >= 0) {
    // layer-0 features: rows r = 0..2rho hold positions t-2rho .. t  (keys then values)
    const int C0 = 2 * D;
    for (int idx = tid; idx < rows0 * C0; idx += kUpdThreads) {
      const int r = idx / C0, m = idx - r * C0;
      const int p = t - 2 * rho + r;
      float x = 0.f;
      if (p >= 0) {
        const bool is_v = m >= D;
        const int mm = is_v ? m - D : m;
        if (p == t) {
          x = to_f32((is_v ? v_new : k_new)[head * D + mm]);
        } else {
          const int64_t row = head * window + (p % window);
          x = to_f32((is_v ? v_win : k_win)[row * D + mm]);
        }
      }
      buf_a[r * lds_row_floats + m] = x;
    }
    __syncthreads();
    float* cur = buf_a;
    float* nxt = buf_b;
    int cur_rows = rows0, cur_lo = t - 2 * rho, cin = C0;
    for (int l = 0; l < cnn.n_layers; ++l) {
      const int ks = cnn.kernel[l], dil = cnn.dilation[l], cout = cnn.c_out[l];
      const int half = dil * (ks - 1) / 2;
      const int out_rows = cur_rows - 2 * half;
      const int out_lo = cur_lo + half;
      const T* W = static_cast<const T*>(cnn.w[l]) + (int64_t)h * cout * cin * ks;
      // kConvSplit adjacent lanes share one (row, channel): each sums a contiguous slice of the input
      // channels over all taps, then the slices are added in a fixed order.
      const int per = (cin + kConvSplit - 1) / kConvSplit;
      for (int idx = tid; idx < out_rows * cout * kConvSplit; idx += kUpdThreads) {
        const int sub = idx % kConvSplit, rc = idx / kConvSplit;
        const int r = rc / cout, c = rc - r * cout;
        float acc = 0.f;
        if (out_lo + r >= 0) {
          const T* Wc = W + (int64_t)c * cin * ks;
          const int m0 = sub * per, m1 = min(cin, m0 + per);
          for (int m = m0; m < m1; ++m)
            for (int tap = 0; tap < ks; ++tap)
              acc = fmaf(cur[(r + tap * dil) * lds_row_floats + m], to_f32(Wc[m * ks + tap]), acc);
        }
#pragma unroll
        for (int off = kConvSplit / 2; off > 0; off >>= 1) acc += __shfl_xor(acc, off, kWave);
        if (sub == 0) {
          // activations at positions before the sequence start are zero padding, not Swish(bias)
          nxt[r * lds_row_floats + c] = (out_lo + r >= 0) ? silu_f32(acc + cnn.bias[l][h * cout + c]) : 0.f;
        }
      }
      __syncthreads();
      float* tmp = cur; cur = nxt; nxt = tmp;
      cur_rows = out_rows; cur_lo = out_lo; cin = cout;
    }
    // cur holds one row (position j_fin) of cin channels
    if (tid < kWave) {
      float part = 0.f;
      for (int c = tid; c < cin; c += kWave) part = fmaf(cur[c], to_f32(static_cast<const T*>(cnn.w_out)[h * cin + c]), part);
      // fixed-order reduction across the wave (deterministic)
      part = wave_sum(part);
      if (tid == 0) win_score[head * window + (j_fin % window)] = part + cnn.b_out[h];
    }
  }

  // ---- 2. eviction of position e = t - window ---------------------------------------------------
  int dst = -1;  // compact slot that receives row e, or -1
  float key_e = 0.f;
  if (e_pos >= 0 && budget > 0) {
    const bool cand = (e_pos < sink) || (z_e > tau);
    key_e = select_key(z_e, e_pos, sink);
    if (cand) {
      if (cnt < budget) {
        dst = cnt;
      } else {
        // worst entry: lowest key, among equal keys the latest position
        unsigned long long best = ~0ull;
        for (int r = tid; r < budget; r += kUpdThreads) {
          const uint32_t u = order_key(ret_score[head * budget + r] + 0.0f);
          const uint32_t pinv = 0xFFFFFFFFu - (uint32_t)ret_pos[head * budget + r];
          const unsigned long long comp = ((unsigned long long)u << 32) | pinv;
          best = comp < best ? comp : best;
        }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) {
          unsigned long long o = __shfl_xor(best, off, kWave);
          best = o < best ? o : best;
        }
        if ((tid & (kWave - 1)) == 0) red[tid / kWave] = best;
        __syncthreads();
        best = red[0];
#pragma unroll
        for (int w = 1; w < kUpdThreads / kWave; ++w) best = red[w] < best ? red[w] : best;
        const uint32_t worst_u = (uint32_t)(best >> 32);
        const int worst_pos = (int)(0xFFFFFFFFu - (uint32_t)(best & 0xFFFFFFFFull));
        if (tid == 0) worst_slot = -1;
        __syncthreads();
        for (int r = tid; r < budget; r += kUpdThreads)
          if (ret_pos[head * budget + r] == worst_pos) worst_slot = r;  // positions are unique
        __syncthreads();
        if (order_key(key_e) > worst_u) dst = worst_slot;
      }
    }
  }

  // ---- 3. move row e into the compact segment, then overwrite its ring slot with token t --------
  __syncthreads();  // every thread has read z_e, cnt and the ring rows it needs
  const int pieces = D * (int)sizeof(T) / 16;
  const int64_t ring_row = (head * window + slot) * D;
  if (dst >= 0) {
    const int64_t ret_row = (head * budget + dst) * D;
    if (tid < pieces) reinterpret_cast<u32x4*>(k_ret + ret_row)[tid] = reinterpret_cast<const u32x4*>(k_win + ring_row)[tid];
    else if (tid < 2 * pieces)
      reinterpret_cast<u32x4*>(v_ret + ret_row)[tid - pieces] = reinterpret_cast<const u32x4*>(v_win + ring_row)[tid - pieces];
    if (tid == 0) {
      ret_score[head * budget + dst] = key_e;
      ret_pos[head * budget + dst] = e_pos;
      if (dst == cnt) ret_count[head] = cnt + 1;
    }
  }
  __syncthreads();
  if (tid < pieces) reinterpret_cast<u32x4*>(k_win + ring_row)[tid] = reinterpret_cast<const u32x4*>(k_new + head * D)[tid];
  else if (tid < 2 * pieces)
    reinterpret_cast<u32x4*>(v_win + ring_row)[tid - pieces] = reinterpret_cast<const u32x4*>(v_new + head * D)[tid - pieces];
}

// --------------------------------------------------------------------------------------------------
// attention partials
// --------------------------------------------------------------------------------------------------
// exp used by the softmax: library expf for fp32 storage (1e-5 tolerance), hardware exp2 path for bf16.
template <typename T> __device__ __forceinline__ float soft_exp(float x);
template <> __device__ __forceinline__ float soft_exp<float>(float x) { return expf(x); }
template <> __device__ __forceinline__ float soft_exp<bf16_t>(float x) { return __expf(x); }

template <typename T> struct Piece;  // 16 bytes of a row as fp32 values
template <> struct Piece<float> {
  static constexpr int N = 4;
  static __device__ __forceinline__ void load(const float* p, float (&x)[4]) {
    const f32x4 r = *reinterpret_cast<const f32x4*>(p);
    x[0] = r[0]; x[1] = r[1]; x[2] = r[2]; x[3] = r[3];
  }
};
template <> struct Piece<bf16_t> {
  static constexpr int N = 8;
  static __device__ __forceinline__ void load(const bf16_t* p, float (&x)[8]) {
    const u32x4 r = *reinterpret_cast<const u32x4*>(p);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      x[2 * i] = __uint_as_float(r[i] << 16);
      x[2 * i + 1] = __uint_as_float(r[i] & 0xFFFF0000u);
    }
  }
};

// Partial record per (sequence, query head, split): [max, sum, acc[D]] floats.
template <typename T, int D>
__global__ void __launch_bounds__(kAttnThreads)
decode_attention_kernel(const T* __restrict__ q, const T* __restrict__ k_win, const T* __restrict__ v_win,
                        const T* __restrict__ k_ret, const T* __restrict__ v_ret,
                        const int32_t* __restrict__ ret_count, const int32_t* __restrict__ n_seen, int Hq, int Hkv,
                        int window, int budget, float scale, int nsplit, float* __restrict__ partial) {
  constexpr int EPL = Piece<T>::N;          // elements per lane
  constexpr int LPR = D / EPL;              // lanes per row
  constexpr int GPW = kWave / LPR;          // row groups per wave
  constexpr int GPB = GPW * (kAttnThreads / kWave);
  constexpr int NW = kAttnThreads / kWave;
  __shared__ float red_m[NW][GPW], red_l[NW][GPW];
  __shared__ float red_acc[NW][GPW][D];

  const int b = blockIdx.x / Hkv, h = blockIdx.x - b * Hkv;
  const int split = blockIdx.y;
  const int64_t head = (int64_t)b * Hkv + h;
  const int G = Hq / Hkv;
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const int sub = lane % LPR, grp = lane / LPR;
  const int t = n_seen[b];                                   // the new token already sits in slot t % window
  const int n_valid = t + 1 < window ? t + 1 : window;
  const int cnt = budget > 0 ? ret_count[head] : 0;
  const int n_rows = n_valid + cnt;
  const int chunk = (n_rows + nsplit - 1) / nsplit;
  const int r_begin = split * chunk;
  const int r_end = r_begin + chunk < n_rows ? r_begin + chunk : n_rows;
  const T* kw = k_win + head * window * D;
  const T* vw = v_win + head * window * D;
  const T* kr = k_ret + head * budget * D;
  const T* vr = v_ret + head * budget * D;

  for (int g = 0; g < G; ++g) {
    const int hq = h * G + g;
    float qf[EPL];
    Piece<T>::load(q + ((int64_t)b * Hq + hq) * D + sub * EPL, qf);
#pragma unroll
    for (int i = 0; i < EPL; ++i) qf[i] *= scale;
    float m_run = -INFINITY, l_run = 0.f, acc[EPL];
#pragma unroll
    for (int i = 0; i < EPL; ++i) acc[i] = 0.f;

    for (int r0 = r_begin + wave * GPW + grp; r0 < r_end; r0 += GPB * kRowsInFlight) {
      float kf[kRowsInFlight][EPL], vf[kRowsInFlight][EPL], s[kRowsInFlight];
#pragma unroll
      for (int u = 0; u < kRowsInFlight; ++u) {
        const int r = r0 + u * GPB;
        if (r < r_end) {
          const T* kp = r < n_valid ? kw + (int64_t)r * D : kr + (int64_t)(r - n_valid) * D;
          const T* vp = r < n_valid ? vw + (int64_t)r * D : vr + (int64_t)(r - n_valid) * D;
          Piece<T>::load(kp + sub * EPL, kf[u]);
          Piece<T>::load(vp + sub * EPL, vf[u]);
        } else {
#pragma unroll
          for (int i = 0; i < EPL; ++i) { kf[u][i] = 0.f; vf[u][i] = 0.f; }
        }
      }
      float m_new = m_run;
#pragma unroll
      for (int u = 0; u < kRowsInFlight; ++u) {
        float d = 0.f;
#pragma unroll
        for (int i = 0; i < EPL; ++i) d = fmaf(qf[i], kf[u][i], d);
#pragma unroll
        for (int off = LPR / 2; off > 0; off >>= 1) d += __shfl_xor(d, off, kWave);
        s[u] = (r0 + u * GPB < r_end) ? d : -INFINITY;
        m_new = fmaxf(m_new, s[u]);
      }
      // r0 < r_end, so row u = 0 is real and m_new is finite
      const float alpha = soft_exp<T>(m_run - m_new);
      l_run *= alpha;
#pragma unroll
      for (int i = 0; i < EPL; ++i) acc[i] *= alpha;
#pragma unroll
      for (int u = 0; u < kRowsInFlight; ++u) {
        const float p = soft_exp<T>(s[u] - m_new);
        l_run += p;
#pragma unroll
        for (int i = 0; i < EPL; ++i) acc[i] = fmaf(p, vf[u][i], acc[i]);
      }
      m_run = m_new;
    }

    // merge the row groups of the block (fixed order -> deterministic)
    if (sub == 0) { red_m[wave][grp] = m_run; red_l[wave][grp] = l_run; }
#pragma unroll
    for (int i = 0; i < EPL; ++i) red_acc[wave][grp][sub * EPL + i] = acc[i];
    __syncthreads();
    if (threadIdx.x < D) {
      float M = -INFINITY;
      for (int w = 0; w < NW; ++w)
        for (int gg = 0; gg < GPW; ++gg) M = fmaxf(M, red_m[w][gg]);
      float L = 0.f, A = 0.f;
      if (M != -INFINITY) {
        for (int w = 0; w < NW; ++w)
          for (int gg = 0; gg < GPW; ++gg) {
            const float f = soft_exp<T>(red_m[w][gg] - M);
            L = fmaf(red_l[w][gg], f, L);
            A = fmaf(red_acc[w][gg][threadIdx.x], f, A);
          }
      }
      float* rec = partial + (((int64_t)b * Hq + hq) * nsplit + split) * (D + 2);
      if (threadIdx.x == 0) { rec[0] = M; rec[1] = L; }
      rec[2 + threadIdx.x] = A;
    }
    __syncthreads();
  }
}

template <typename T, int D>
__global__ void __launch_bounds__(D)
decode_combine_kernel(const float* __restrict__ partial, int nsplit, int Hq, int rho, T* __restrict__ out,
                      int32_t* __restrict__ n_seen, int32_t* __restrict__ n_scored) {
  const int64_t bh = blockIdx.x;  // b * Hq + hq
  const float* rec = partial + bh * nsplit * (D + 2);
  float M = -INFINITY;
  for (int s = 0; s < nsplit; ++s) M = fmaxf(M, rec[s * (D + 2)]);
  float L = 0.f, A = 0.f;
  for (int s = 0; s < nsplit; ++s) {
    const float m = rec[s * (D + 2)];
    if (m == -INFINITY) continue;
    const float f = soft_exp<T>(m - M);
    L = fmaf(rec[s * (D + 2) + 1], f, L);
    A = fmaf(rec[s * (D + 2) + 2 + threadIdx.x], f, A);
  }
  out[bh * D + threadIdx.x] = from_f32<T>(A / L);
  if (threadIdx.x == 0 && bh % Hq == 0) {
    const int b = (int)(bh / Hq);
    const int t1 = n_seen[b] + 1;
    n_seen[b] = t1;
    n_scored[b] = t1 > rho ? t1 - rho : 0;
  }
}

template <typename T, int D>
hipError_t run(const ltea_cfg& cfg, const ltea_cnn& cnn, const void* q, const void* k, const void* v, void* out,
               const ltea_cache& c, int n_seqs, void* workspace, hipStream_t stream) {
  const int rho = cnn_rho(&cnn);
  CnnDev cd;
  cd.n_layers = cnn.n_layers;
  int row_floats = 2 * cfg.D;
  for (int l = 0; l < LTEA_MAX_CNN_LAYERS; ++l) {
    const bool on = l < cnn.n_layers;
    cd.kernel[l] = on ? cnn.kernel[l] : 1;
    cd.dilation[l] = on ? cnn.dilation[l] : 1;
    cd.c_out[l] = on ? cnn.c_out[l] : 0;
    cd.w[l] = on ? cnn.w[l] : nullptr;
    cd.bias[l] = on ? cnn.bias[l] : nullptr;
    if (on && cnn.c_out[l] > row_floats) row_floats = cnn.c_out[l];
  }
  cd.w_out = cnn.w_out;
  cd.b_out = cnn.b_out;
  const size_t lds_bytes = (size_t)2 * (2 * rho + 1) * row_floats * sizeof(float);
  const unsigned heads = (unsigned)n_seqs * (unsigned)cfg.Hkv;
  hipLaunchKernelGGL(decode_update_kernel<T>, dim3(heads), dim3(kUpdThreads), lds_bytes, stream, cd, rho, row_floats,
                     static_cast<const T*>(k), static_cast<const T*>(v), cfg.Hkv, cfg.D, cfg.window, cfg.budget,
                     cfg.sink, cfg.tau_logit, static_cast<T*>(c.k_win), static_cast<T*>(c.v_win), c.win_score,
                     static_cast<T*>(c.k_ret), static_cast<T*>(c.v_ret), c.ret_score, c.ret_pos, c.ret_count,
                     c.n_seen);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const int nsplit = decode_num_splits(cfg, n_seqs);
  const float scale = cfg.softmax_scale > 0.f ? cfg.softmax_scale : 1.0f / sqrtf((float)cfg.D);
  float* partial = static_cast<float*>(workspace);
  hipLaunchKernelGGL((decode_attention_kernel<T, D>), dim3(heads, (unsigned)nsplit), dim3(kAttnThreads), 0, stream,
                     static_cast<const T*>(q), static_cast<const T*>(c.k_win), static_cast<const T*>(c.v_win),
                     static_cast<const T*>(c.k_ret), static_cast<const T*>(c.v_ret), c.ret_count, c.n_seen, cfg.Hq,
                     cfg.Hkv, cfg.window, cfg.budget, scale, nsplit, partial);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((decode_combine_kernel<T, D>), dim3((unsigned)n_seqs * (unsigned)cfg.Hq), dim3(D), 0, stream,
                     partial, nsplit, cfg.Hq, rho, static_cast<T*>(out), c.n_seen, c.n_scored);
  return hipGetLastError();
}

}  // namespace

int decode_num_splits(const ltea_cfg& cfg, int n_seqs) {
  const long heads = (long)n_seqs * cfg.Hkv;
  const int rows = cfg.window + cfg.budget;
  int by_fill = (int)((2048 + heads - 1) / (heads > 0 ? heads : 1));  // aim for >= 2048 workgroups
  int by_rows = (rows + 127) / 128;                                   // at least 128 rows per split
  int n = by_fill < by_rows ? by_fill : by_rows;
  if (n < 1) n = 1;
  if (n > 64) n = 64;
  return n;
}

size_t decode_workspace(const ltea_cfg& cfg, int n_seqs) {
  return (size_t)n_seqs * cfg.Hq * decode_num_splits(cfg, n_seqs) * (cfg.D + 2) * sizeof(float);
}

size_t decode_update_lds_bytes(const ltea_cfg& cfg, const ltea_cnn& cnn) {
  int row_floats = 2 * cfg.D;
  for (int l = 0; l < cnn.n_layers; ++l) row_floats = cnn.c_out[l] > row_floats ? cnn.c_out[l] : row_floats;
  return (size_t)2 * (2 * cnn_rho(&cnn) + 1) * row_floats * sizeof(float);
}

hipError_t launch_decode_step(const ltea_cfg& cfg, const ltea_cnn& cnn, const void* q, const void* k, const void* v,
                              void* out, const ltea_cache& c, int n_seqs, void* workspace, hipStream_t stream) {
  if (n_seqs == 0) return hipSuccess;
  if (cfg.dtype == LTEA_F32) {
    return cfg.D == 64 ? run<float, 64>(cfg, cnn, q, k, v, out, c, n_seqs, workspace, stream)
                       : run<float, 128>(cfg, cnn, q, k, v, out, c, n_seqs, workspace, stream);
  }
  return cfg.D == 64 ? run<bf16_t, 64>(cfg, cnn, q, k, v, out, c, n_seqs, workspace, stream)
                     : run<bf16_t, 128>(cfg, cnn, q, k, v, out, c, n_seqs, workspace, stream);
}

}  // namespace ltea
