// One decode step of the SWA+LTE cache (paper Section 3.1.3: cache replacement, decode attention and
// the deferred scoring of Section 3.1.1 item 2).
//
// Two launches per step on the caller's stream:
//
//   decode_main_kernel    1-D grid = [scoring workgroups][attention workgroups].  Nothing in the cache is modified.
//     scoring role        finalises the logit of position t-rho of every (sequence, KV head) from the 2*rho newest
//                         ring rows plus the incoming token, and parks it in the workspace.  Single-layer bf16:
//                         one workgroup per (KV head, 64 sequences); the conv over the batch is a small GEMM
//                         [sequences x taps*2D] . [taps*2D x C] on v_mfma_f32_16x16x32_bf16 with both operands
//                         read straight from global memory (weights are shared by all sequences of a head).
//                         Multi-layer bf16 (given the larger workspace): a packing role of this launch (one
//                         workgroup per sequence) copies the receptive-field windows of all sequences into the
//                         workspace as tiny sequences; the fused prefill scoring kernel runs over them between
//                         this launch and the finishing one, which picks each window's centre logit.
//                         Otherwise (fp32, unusual stacks): one workgroup per (sequence, head), activation pyramid
//                         in LDS.  These few workgroups are dispatched first and hide under the streaming.
//     attention role      the memory-bound part: grid (sequence x KV head) x splits; each workgroup streams its
//                         share of the rows the query must see AFTER this step's cache update, without waiting
//                         for that update: the row of ring slot t % window is taken from the incoming k_t, v_t,
//                         and the compact slot that will receive the evicted token (decided from the old state:
//                         one pass over `budget` keys, only by workgroups whose share touches the compact
//                         segment) is taken from the old ring row.  16-byte loads, one row per D*sizeof(T)/16
//                         lanes, several rows in flight per lane group, online softmax per group, fixed-order
//                         merges.  Up to four query heads of a KV group share one pass over the rows.
//   decode_finish_kernel  one workgroup per (sequence, KV head): repeats the eviction decision, moves the evicted
//                         row into the compact segment, writes k_t, v_t and the new logit into the ring, merges
//                         the split partials of the group's query heads into the output row and advances
//                         n_seen / n_scored.
//
// The lazy step (Section 3.1.3, lazy scoring) is the same pair of launches without a scoring role: logits are
// produced between steps by the batched scoring of lazy.hip, the finishing launch leaves n_scored alone and flags a
// token that leaves the window unscored.
#include <string.h>

#include <type_traits>

#include "ltea_common.h"
#include "ltea_kernels.h"
#include "rope_dev.h"

namespace ltea {
namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / kWave;
constexpr int kConvSplit = 8;     // lanes cooperating on one conv output in the scoring role
constexpr int kRowsInFlight = 4;  // rows per lane group per iteration of the streaming loop

struct CnnDev {
  int n_layers;
  int kernel[LTEA_MAX_CNN_LAYERS], dilation[LTEA_MAX_CNN_LAYERS], c_out[LTEA_MAX_CNN_LAYERS];
  const void* w[LTEA_MAX_CNN_LAYERS];
  const float* bias[LTEA_MAX_CNN_LAYERS];
  const void* w_out;
  const float* b_out;
};

struct CacheDev {
  void *k_win, *v_win;
  float* win_score;
  void *k_ret, *v_ret;
  float* ret_score;
  int32_t *ret_pos, *ret_count, *n_seen, *n_scored;
};

struct StepParams {
  int B, Hq, Hkv, D, window, budget, sink, rho, nsplit, lds_row_floats, n_score_blocks, score_mfma;
  float tau, scale;
  // Scores computed before this launch over packed receptive-field windows (multi-layer bf16 CNN): the window of
  // sequence b occupies rows b*(2*rho+1) .. of pre_logits[h][.], its first row is position max(0, t - 2*rho).
  const float* pre_logits;
  int64_t pre_total;
  int pre_stride;            // rows per sequence in pre_logits (2*rho+1, or more when the windows are packed with gaps)
  // packing role of the main launch (multi-layer bf16 CNN): where the windows go; n_pack_blocks = 0 switches it off
  void* pk_k; void* pk_v; int32_t* pk_cu2; uint8_t* pk_row_valid; int n_pack_blocks;
  // Lazy mode (scores come from separate batched launches between steps): nothing is scored here, n_scored is
  // left alone, and a token that leaves the window without a final logit is reported through `status`.
  int lazy;
  int32_t* status;
};

// exp used by the softmax: library expf for fp32 storage (1e-5 tolerance), hardware exp2 path for bf16.
template <typename T> __device__ __forceinline__ float soft_exp(float x);
template <> __device__ __forceinline__ float soft_exp<float>(float x) { return expf(x); }
template <> __device__ __forceinline__ float soft_exp<bf16_t>(float x) { return __expf(x); }

template <typename T> struct Piece;  // 16 bytes of a row as fp32 values
template <> struct Piece<float> {
  static constexpr int N = 4;
  static __device__ __forceinline__ void unpack(const u32x4& r, float (&x)[4]) {
#pragma unroll
    for (int i = 0; i < 4; ++i) x[i] = __uint_as_float(r[i]);
  }
  static __device__ __forceinline__ void load(const float* p, float (&x)[4]) {
    const f32x4 r = *reinterpret_cast<const f32x4*>(p);
    x[0] = r[0]; x[1] = r[1]; x[2] = r[2]; x[3] = r[3];
  }
};
template <> struct Piece<bf16_t> {
  static constexpr int N = 8;
  static __device__ __forceinline__ void unpack(const u32x4& r, float (&x)[8]) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      x[2 * i] = __uint_as_float(r[i] << 16);
      x[2 * i + 1] = __uint_as_float(r[i] & 0xFFFF0000u);
    }
  }
  static __device__ __forceinline__ void load(const bf16_t* p, float (&x)[8]) {
    const u32x4 r = *reinterpret_cast<const u32x4*>(p);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      x[2 * i] = __uint_as_float(r[i] << 16);
      x[2 * i + 1] = __uint_as_float(r[i] & 0xFFFF0000u);
    }
  }
};

// Where does the token leaving the window go?  Returns the compact slot that receives it (== cnt for an
// append), or -1 if it is dropped.  A pure function of the state before the step, evaluated identically by
// every workgroup that needs it.  All threads of the block must call it; `red`/`slot_out` are LDS scratch.
__device__ __forceinline__ int eviction_target(int t, int window, int budget, int sink, float tau, int cnt,
                                               float z_e, const float* __restrict__ ret_score,
                                               const int32_t* __restrict__ ret_pos, unsigned long long* red,
                                               int* slot_out) {
  const int e_pos = t - window;
  if (e_pos < 0 || budget <= 0) return -1;
  if (!((e_pos < sink) || (z_e > tau))) return -1;
  if (cnt < budget) return cnt;
  // victim: lowest key, among equal keys the latest position
  const int tid = threadIdx.x;
  unsigned long long best = ~0ull;
  for (int r = tid; r < budget; r += kThreads) {
    const uint32_t u = order_key(ret_score[r] + 0.0f);
    const uint32_t pinv = 0xFFFFFFFFu - (uint32_t)ret_pos[r];
    const unsigned long long comp = ((unsigned long long)u << 32) | pinv;
    best = comp < best ? comp : best;
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    const unsigned long long o = __shfl_xor(best, off, kWave);
    best = o < best ? o : best;
  }
  __syncthreads();
  if ((tid & (kWave - 1)) == 0) red[tid / kWave] = best;
  if (tid == 0) *slot_out = -1;
  __syncthreads();
  best = red[0];
#pragma unroll
  for (int w = 1; w < kWaves; ++w) best = red[w] < best ? red[w] : best;
  const uint32_t worst_u = (uint32_t)(best >> 32);
  const int worst_pos = (int)(0xFFFFFFFFu - (uint32_t)(best & 0xFFFFFFFFull));
  for (int r = tid; r < budget; r += kThreads)
    if (ret_pos[r] == worst_pos) *slot_out = r;  // positions are unique
  __syncthreads();
  const int victim = *slot_out;
  return order_key(select_key(z_e, e_pos, sink)) > worst_u ? victim : -1;
}

// ---- scoring role ------------------------------------------------------------------------------------------
template <typename T>
__device__ __forceinline__ void score_new_token(const CnnDev& cnn, const StepParams& P, const T* __restrict__ k_new,
                                                const T* __restrict__ v_new, const T* __restrict__ k_win,
                                                const T* __restrict__ v_win, int64_t head, int h, int t, float* lds,
                                                float* __restrict__ ws_logit) {
  const int tid = threadIdx.x;
  const int rho = P.rho, D = P.D, window = P.window, row_f = P.lds_row_floats;
  const int j_fin = t - rho;
  if (j_fin < 0) return;
  const int rows0 = 2 * rho + 1;
  float* cur = lds;
  float* nxt = lds + (size_t)rows0 * row_f;
  // layer-0 features: rows r = 0..2rho hold positions t-2rho .. t  (keys then values), one 16-byte piece per
  // thread per pass so that the whole staging costs one memory round trip
  const int C0 = 2 * D;
  constexpr int EPP = 16 / (int)sizeof(T);  // elements per piece
  const int ppr = C0 / EPP;
  for (int idx = tid; idx < rows0 * ppr; idx += kThreads) {
    const int r = idx / ppr, piece = idx - r * ppr;
    const int m = piece * EPP;
    const int p = t - 2 * rho + r;
    float x[EPP];
#pragma unroll
    for (int i = 0; i < EPP; ++i) x[i] = 0.f;
    if (p >= 0) {
      const bool is_v = m >= D;
      const int mm = is_v ? m - D : m;
      const T* src = (p == t) ? (is_v ? v_new : k_new) + head * D + mm
                              : (is_v ? v_win : k_win) + (head * window + (p % window)) * D + mm;
      Piece<T>::load(src, x);
    }
#pragma unroll
    for (int i = 0; i < EPP; ++i) cur[r * row_f + m + i] = x[i];
  }
  __syncthreads();
  int cur_rows = rows0, cur_lo = t - 2 * rho, cin = C0;
  for (int l = 0; l < cnn.n_layers; ++l) {
    const int ks = cnn.kernel[l], dil = cnn.dilation[l], cout = cnn.c_out[l];
    const int half = dil * (ks - 1) / 2;
    const int out_rows = cur_rows - 2 * half;
    const int out_lo = cur_lo + half;
    const T* W = static_cast<const T*>(cnn.w[l]) + (int64_t)h * cout * cin * ks;
    // kConvSplit adjacent lanes share one (row, channel): each sums a contiguous slice of the input channels
    // over all taps (a contiguous run of weights), then the slices are added in a fixed order.
    const int per = (cin + kConvSplit - 1) / kConvSplit;
    for (int idx = tid; idx < out_rows * cout * kConvSplit; idx += kThreads) {
      const int sub = idx % kConvSplit, rc = idx / kConvSplit;
      const int r = rc / cout, c = rc - r * cout;
      float acc = 0.f;
      if (out_lo + r >= 0) {
        const int m0 = sub * per, m1 = min(cin, m0 + per);
        const T* Wc = W + ((int64_t)c * cin + m0) * ks;           // weights of (c, m0.., all taps): contiguous
        const float* xin = cur + r * row_f;
        const int n_el = (m1 - m0) * ks;
        int e = 0;
        if constexpr (sizeof(T) == 2) {
          if ((reinterpret_cast<uintptr_t>(Wc) & 15u) == 0) {
            // 16-byte weight loads in register-double-buffered batches: the slice costs about one memory round
            // trip instead of one per load
            constexpr int VB = 2;
            const int n_batches = n_el / (8 * VB);
            u32x4 wcur[VB], wnxt[VB];
            if (n_batches > 0) {
#pragma unroll
              for (int i = 0; i < VB; ++i) wcur[i] = *reinterpret_cast<const u32x4*>(Wc + 8 * i);
            }
            int m = m0, tap = 0;
            for (int bt = 0; bt < n_batches; ++bt) {
              if (bt + 1 < n_batches) {
#pragma unroll
                for (int i = 0; i < VB; ++i) wnxt[i] = *reinterpret_cast<const u32x4*>(Wc + (bt + 1) * 8 * VB + 8 * i);
              }
#pragma unroll
              for (int i = 0; i < VB; ++i) {
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                  const float wf = (j & 1) ? __uint_as_float(wcur[i][j / 2] & 0xFFFF0000u) : __uint_as_float(wcur[i][j / 2] << 16);
                  acc = fmaf(xin[tap * dil * row_f + m], wf, acc);
                  if (++tap == ks) { tap = 0; ++m; }
                }
              }
#pragma unroll
              for (int i = 0; i < VB; ++i) wcur[i] = wnxt[i];
            }
            e = n_batches * 8 * VB;
          }
        }
        for (; e < n_el; ++e) {
          const int m = m0 + e / ks, tap = e % ks;
          acc = fmaf(xin[tap * dil * row_f + m], to_f32(Wc[e]), acc);
        }
      }
#pragma unroll
      for (int off = kConvSplit / 2; off > 0; off >>= 1) acc += __shfl_xor(acc, off, kWave);
      if (sub == 0) {
        // activations at positions before the sequence start are zero padding, not Swish(bias)
        nxt[r * row_f + c] = (out_lo + r >= 0) ? silu_f32(acc + cnn.bias[l][h * cout + c]) : 0.f;
      }
    }
    __syncthreads();
    float* tmp = cur; cur = nxt; nxt = tmp;
    cur_rows = out_rows; cur_lo = out_lo; cin = cout;
  }
  // cur holds one row (position j_fin) of cin channels
  if (tid < kWave) {
    float part = 0.f;
    for (int c = tid; c < cin; c += kWave)
      part = fmaf(cur[c], to_f32(static_cast<const T*>(cnn.w_out)[h * cin + c]), part);
    part = wave_sum(part);  // fixed order: deterministic
    if (tid == 0) ws_logit[head] = part + cnn.b_out[h];
  }
}

// ---- scoring role, batched over sequences on MFMA (single conv layer, bf16, kernel size KS) ----------------------
// Workgroup = (KV head h, group of 64 sequences).  The conv over the batch is the GEMM
//   out[sequence, channel] = sum_{tap, m} x[sequence][tap][m] * W[channel][m][tap]
// on v_mfma_f32_16x16x32_bf16: 4 row tiles of 16 sequences, 2 column tiles of 16 channels, K = (tap, m) with 32
// input channels per instruction.  The four waves split the input channels, so every weight is fetched once per
// workgroup (KS contiguous 16-byte loads per lane cover all taps of its 8 channels) and reused for all row tiles;
// features come straight from the ring rows / the incoming token.  Partial sums of the waves meet in LDS.
// Lane roles: A row / B column = lane % 16, K group kg = lane / 16 supplies 8 consecutive channels;
// accumulator register r of a lane is (row 4*kg + r, column lane % 16).
template <int D, int KS>
__device__ __forceinline__ void score_new_tokens_mfma(const CnnDev& cnn, const StepParams& P, const CacheDev& C,
                                                      const bf16_t* __restrict__ k_new, const bf16_t* __restrict__ v_new,
                                                      int h, int b0, float* red /* 2048 floats of LDS */,
                                                      float* __restrict__ ws_logit, int32_t* __restrict__ ws_t) {
  constexpr int C2 = 2 * D;
  constexpr int MCW = C2 / 32 / kWaves;  // 32-channel chunks per wave
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid / kWave;
  const int row = lane & 15, kg = lane >> 4;
  const int dil = cnn.dilation[0], Cout = cnn.c_out[0];
  const int rho = P.rho, window = P.window;
  const uint16_t* W = reinterpret_cast<const uint16_t*>(cnn.w[0]) + (int64_t)h * Cout * C2 * KS;

  const int seq_l = tid / 16, chp = tid % 16;   // finishing thread: sequence seq_l of a row tile, channels chp, chp+16
  float bias0 = 0.f, bias1 = 0.f, wo0 = 0.f, wo1 = 0.f;
  if (chp < Cout) { bias0 = cnn.bias[0][h * Cout + chp]; wo0 = to_f32(static_cast<const bf16_t*>(cnn.w_out)[h * Cout + chp]); }
  if (chp + 16 < Cout) { bias1 = cnn.bias[0][h * Cout + chp + 16]; wo1 = to_f32(static_cast<const bf16_t*>(cnn.w_out)[h * Cout + chp + 16]); }

  // two row tiles (32 sequences) per pass keeps the register footprint of this role below the streaming role's
#pragma unroll 1
  for (int mt0 = 0; mt0 < 4; mt0 += 2) {
    if (b0 + 16 * mt0 >= P.B) break;   // uniform: no sequences left
    int t_mt[2];
    const bf16_t *kw_mt[2], *vw_mt[2], *kn_mt[2], *vn_mt[2];
    bool ok_mt[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int b = b0 + 16 * (mt0 + i) + row;
      ok_mt[i] = b < P.B;
      const int bc = ok_mt[i] ? b : P.B - 1;
      const int64_t head = (int64_t)bc * P.Hkv + h;
      t_mt[i] = C.n_seen[bc];
      kw_mt[i] = static_cast<const bf16_t*>(C.k_win) + head * window * D;
      vw_mt[i] = static_cast<const bf16_t*>(C.v_win) + head * window * D;
      kn_mt[i] = k_new + head * D;
      vn_mt[i] = v_new + head * D;
      if (h == 0 && wv == 0 && kg == 0 && ok_mt[i]) ws_t[b] = t_mt[i];
    }
    f32x4 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int nb = 0; nb < 2; ++nb) acc[i][nb] = f32x4{0.f, 0.f, 0.f, 0.f};

#pragma unroll 1
    for (int mcw = 0; mcw < MCW; ++mcw) {
      const int m = 32 * (wv * MCW + mcw) + 8 * kg;   // first of this lane's 8 input channels
      // weights of channels m..m+7, all taps, for output channels row and 16+row: KS*8 contiguous elements each
      uint32_t wraw[2][KS * 4];
#pragma unroll
      for (int nb = 0; nb < 2; ++nb) {
        const int c = 16 * nb + row;
        const u32x4* wp = reinterpret_cast<const u32x4*>(W + ((int64_t)(c < Cout ? c : 0) * C2 + m) * KS);
#pragma unroll
        for (int i = 0; i < KS; ++i) {
          u32x4 x = wp[i];
          if (c >= Cout) x = u32x4{0u, 0u, 0u, 0u};
          wraw[nb][4 * i] = x[0]; wraw[nb][4 * i + 1] = x[1]; wraw[nb][4 * i + 2] = x[2]; wraw[nb][4 * i + 3] = x[3];
        }
      }
#pragma unroll
      for (int tap = 0; tap < KS; ++tap) {
        // B operand: element e is flat index e*KS + tap of the lane's weight run
        u32x4 bop[2];
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
#pragma unroll
          for (int e2 = 0; e2 < 4; ++e2) {
            const int f0 = (2 * e2) * KS + tap, f1 = (2 * e2 + 1) * KS + tap;
            const uint32_t lo16 = (f0 & 1) ? (wraw[nb][f0 / 2] >> 16) : (wraw[nb][f0 / 2] & 0xFFFFu);
            const uint32_t hi16 = (f1 & 1) ? (wraw[nb][f1 / 2] & 0xFFFF0000u) : (wraw[nb][f1 / 2] << 16);
            bop[nb][e2] = lo16 | hi16;
          }
#pragma unroll
        for (int i = 0; i < 2; ++i) {
          const int p = t_mt[i] - 2 * rho + tap * dil;   // position this tap reads for the token t - rho
          const bool p_ok = p >= 0 && ok_mt[i];
          const int slot_p = (p_ok ? p : 0) % window;
          const bf16_t* src;
          if (m < D) src = (p == t_mt[i] ? kn_mt[i] : kw_mt[i] + (int64_t)slot_p * D) + m;
          else src = (p == t_mt[i] ? vn_mt[i] : vw_mt[i] + (int64_t)slot_p * D) + (m - D);
          u32x4 araw = *reinterpret_cast<const u32x4*>(src);
          if (!p_ok) araw = u32x4{0u, 0u, 0u, 0u};
          const bf16x8 a = __builtin_bit_cast(bf16x8, araw);
          acc[i][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, __builtin_bit_cast(bf16x8, bop[0]), acc[i][0], 0, 0, 0);
          acc[i][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, __builtin_bit_cast(bf16x8, bop[1]), acc[i][1], 0, 0, 0);
        }
      }
    }
    // cross-wave sum, bias, Swish, output projection: one row tile (16 sequences x 32 channels) per round
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      __syncthreads();
#pragma unroll
      for (int nb = 0; nb < 2; ++nb)
#pragma unroll
        for (int r = 0; r < 4; ++r) red[(wv * 16 + 4 * kg + r) * 32 + 16 * nb + row] = acc[i][nb][r];
      __syncthreads();
      float y0 = bias0, y1 = bias1;
#pragma unroll
      for (int w = 0; w < kWaves; ++w) {
        y0 += red[(w * 16 + seq_l) * 32 + chp];
        y1 += red[(w * 16 + seq_l) * 32 + 16 + chp];
      }
      float z = y0 * __frcp_rn(1.0f + __expf(-y0)) * wo0 + y1 * __frcp_rn(1.0f + __expf(-y1)) * wo1;
#pragma unroll
      for (int off = 8; off > 0; off >>= 1) z += __shfl_xor(z, off, kWave);
      const int bb = b0 + 16 * (mt0 + i) + seq_l;
      if (chp == 0 && bb < P.B && C.n_seen[bb] - rho >= 0) ws_logit[(int64_t)bb * P.Hkv + h] = z + cnn.b_out[h];
    }
  }
}

// Receptive-field windows of the token being finalised, packed for the prefill scoring kernels: sequence b gets
// rows b*R .. b*R + len - 1 (R = 2*rho + 1) holding positions max(0, t - 2*rho) .. t (the ring rows and, last, the
// incoming token); a second, possibly empty pseudo-sequence covers the unused rest of the R rows so that the packing
// stays contiguous without a prefix sum over the batch: cu2[2b] = b*R, cu2[2b+1] = b*R + len, cu2[2B] = B*R.
// Rotary models (rope.cos != null): the ring holds rotated keys, which are rotated back here; the incoming token's
// scoring key is kf_new when given, else k_new rotated back at position t.
// One workgroup of 256 threads per sequence b.  ROT = false compiles the rotary branch out (the main launch's packing role).
template <typename T, bool ROT>
__device__ __forceinline__ void pack_window(const CacheDev& C, const T* __restrict__ k_new, const T* __restrict__ v_new,
                                            const T* __restrict__ kf_new, const RopeDev& rope, int32_t* __restrict__ status,
                                            T* __restrict__ win_k, T* __restrict__ win_v, int32_t* __restrict__ cu2, int B,
                                            int Hkv, int D, int window, int rho, int stride_rows,
                                            uint8_t* __restrict__ row_valid, int b) {
  constexpr int EPP = Elems<T>::N;
  const int R = stride_rows;     // 2*rho + 1, or more: windows mode (row_valid given), the rows in between are zeros
  const int t = C.n_seen[b];
  const int first = t - 2 * rho > 0 ? t - 2 * rho : 0;
  const int len = t - first + 1;
  const int pieces = D / EPP;                                 // 16-byte pieces per row
  if (row_valid == nullptr) {
    if (threadIdx.x == 0) {
      cu2[2 * b] = b * R;
      cu2[2 * b + 1] = b * R + len;
      if (b == B - 1) cu2[2 * B] = B * R;
    }
  } else {
    // one sequence of B * R rows; which rows are tokens is said per row, and the others are cleared
    if (threadIdx.x == 0 && b == 0) { cu2[0] = 0; cu2[1] = B * R; }
    for (int r = threadIdx.x; r < R; r += 256) row_valid[b * R + r] = r < len ? 1 : 0;
    const int gap = (R - len) * Hkv * pieces;
    const int64_t dst0 = (int64_t)(b * R + len) * Hkv * D;
    const u32x4 zero4 = {0u, 0u, 0u, 0u};
    for (int i = threadIdx.x; i < gap; i += 256) {
      reinterpret_cast<u32x4*>(win_k + dst0)[i] = zero4;
      reinterpret_cast<u32x4*>(win_v + dst0)[i] = zero4;
    }
  }
  const int items = len * Hkv * pieces;
  bool out_of_tables = false;
  for (int i = threadIdx.x; i < items; i += 256) {
    const int pc = i % pieces, h = (i / pieces) % Hkv, r = i / (pieces * Hkv);
    const int p = first + r;
    const int64_t head = (int64_t)b * Hkv + h;
    const T* sk = p == t ? k_new + head * D : static_cast<const T*>(C.k_win) + (head * window + p % window) * D;
    const T* sv = p == t ? v_new + head * D : static_cast<const T*>(C.v_win) + (head * window + p % window) * D;
    const int64_t dst = ((int64_t)(b * R + r) * Hkv + h) * D;
    u32x4 xk = reinterpret_cast<const u32x4*>(sk)[pc];
    if constexpr (ROT) {
      if (p == t && kf_new != nullptr) {
        xk = reinterpret_cast<const u32x4*>(kf_new + head * D)[pc];
      } else if (rope.cos != nullptr && pc * EPP < rope.rot_dim) {
        if (p >= rope.n_pos) out_of_tables = true;
        else xk = unrotate_piece<T>(rope, p, pc * EPP, xk, sk);
      }
    }
    reinterpret_cast<u32x4*>(win_k + dst)[pc] = xk;
    reinterpret_cast<u32x4*>(win_v + dst)[pc] = reinterpret_cast<const u32x4*>(sv)[pc];
  }
  if (out_of_tables && status != nullptr) atomicOr(status, LTEA_ROPE_RANGE);
}

template <typename T>
__global__ void __launch_bounds__(256)
decode_windows_kernel(CacheDev C, const T* __restrict__ k_new, const T* __restrict__ v_new, const T* __restrict__ kf_new,
                      RopeDev rope, int32_t* __restrict__ status, T* __restrict__ win_k, T* __restrict__ win_v,
                      int32_t* __restrict__ cu2, int B, int Hkv, int D, int window, int rho, int stride_rows,
                      uint8_t* __restrict__ row_valid) {
  pack_window<T, true>(C, k_new, v_new, kf_new, rope, status, win_k, win_v, cu2, B, Hkv, D, window, rho, stride_rows,
                       row_valid, (int)blockIdx.x);
}

// Partial record per (sequence, query head, split): [max, sum, acc[D]] floats.
// GT = query heads of a KV group handled per pass over the rows (1, 2 or 4): every K/V row is loaded once per pass
// and used for GT queries, so grouped-query configurations do not re-stream the cache once per query head.
// SK = kernel size of the batched MFMA scoring role compiled into this instance (3, 5 or 7), 0 for none: the role's
// register needs grow with the kernel size, and one instance holding all three would carry the largest one's spills.
template <typename T, int D, int GT, int SK>
__global__ void __launch_bounds__(kThreads, 4)
decode_main_kernel(CnnDev cnn, CacheDev C, StepParams P, const T* __restrict__ q, const T* __restrict__ k_new,
                   const T* __restrict__ v_new, float* __restrict__ partial, float* __restrict__ ws_logit,
                   int32_t* __restrict__ ws_t, int32_t* __restrict__ ws_dst) {
  constexpr int EPL = Piece<T>::N;  // elements per lane
  constexpr int LPR = D / EPL;      // lanes per row
  constexpr int GPW = kWave / LPR;  // row groups per wave
  constexpr int GPB = GPW * kWaves;
  extern __shared__ float dyn_lds[];  // per-head scoring role: two activation buffers of (2*rho+1) rows
  __shared__ float red_m[kWaves][GPW], red_l[kWaves][GPW];
  __shared__ float red_acc[kWaves][GPW][D];
  __shared__ unsigned long long red64[kWaves];
  __shared__ int slot_lds;

  const int Hkv = P.Hkv, window = P.window, budget = P.budget;
  if ((int)blockIdx.x < P.n_score_blocks) {
    if (P.lazy || P.pre_logits != nullptr) {
      // only the snapshot of the token counts that the finishing launch reads (logits scored outside this launch
      // are picked up by the finishing launch itself, so nothing here waits for them)
      const int b = blockIdx.x * kThreads + threadIdx.x;
      if (b < P.B) ws_t[b] = C.n_seen[b];
      return;
    }
    if constexpr (sizeof(T) == 2 && SK > 0) {
      if (P.score_mfma) {   // == SK (the launcher picks the instance)
        const int h = blockIdx.x % Hkv, sg = blockIdx.x / Hkv;
        float* red = &red_acc[0][0][0];
        static_assert(sizeof(red_acc) >= 2048 * sizeof(float), "cross-wave scoring sums need 2048 floats");
        score_new_tokens_mfma<D, SK>(cnn, P, C, k_new, v_new, h, 64 * sg, red, ws_logit, ws_t);
        return;
      }
    }
    const int b = blockIdx.x / Hkv, h = blockIdx.x - b * Hkv;
    const int t = C.n_seen[b];
    if (h == 0 && threadIdx.x == 0) ws_t[b] = t;
    score_new_token<T>(cnn, P, k_new, v_new, static_cast<const T*>(C.k_win), static_cast<const T*>(C.v_win),
                       (int64_t)b * Hkv + h, h, t, dyn_lds, ws_logit);
    return;
  }
  if ((int)blockIdx.x < P.n_score_blocks + P.n_pack_blocks) {
    // packing role (multi-layer bf16 CNN): one workgroup per sequence copies the receptive-field window of the token
    // being finalised into the buffers that the scoring launch between this one and the finishing one reads
    if constexpr (sizeof(T) == 2)
      pack_window<T, false>(C, k_new, v_new, nullptr, RopeDev{}, nullptr, static_cast<T*>(P.pk_k), static_cast<T*>(P.pk_v),
                            P.pk_cu2, P.B, Hkv, D, window, P.rho, P.pre_stride, P.pk_row_valid,
                            (int)blockIdx.x - P.n_score_blocks);
    return;
  }
  const int work = blockIdx.x - P.n_score_blocks - P.n_pack_blocks;
  const int nsplit = P.nsplit;
  const int split = work % nsplit;
  const int64_t head = work / nsplit;
  const int b = (int)(head / Hkv), h = (int)(head - (int64_t)b * Hkv);
  const int t = C.n_seen[b];
  const T* kw = static_cast<const T*>(C.k_win) + head * window * D;
  const T* vw = static_cast<const T*>(C.v_win) + head * window * D;
  const int G = P.Hq / Hkv;
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const int sub = lane % LPR, grp = lane / LPR;
  const T* kr = static_cast<const T*>(C.k_ret) + head * budget * D;
  const T* vr = static_cast<const T*>(C.v_ret) + head * budget * D;
  const T* kn = k_new + head * D;
  const T* vn = v_new + head * D;

  // The state after this step, described from the state before it.  Rows are addressed in a fixed slot space
  // [ring slots 0..window) ++ [compact slots 0..budget) split evenly, so a workgroup whose share holds ring
  // slots only never needs the eviction decision (one pass over `budget` keys plus three barriers).
  const int slot = t % window;
  const int n_valid = t + 1 < window ? t + 1 : window;
  const int chunk = (window + budget + nsplit - 1) / nsplit;
  const int r_begin = split * chunk;
  const int r_end = r_begin + chunk < window + budget ? r_begin + chunk : window + budget;
  int dst = -1, cnt = 0;
  if (r_end > window && budget > 0) {   // uniform across the workgroup
    const int cnt_old = C.ret_count[head];
    const float z_e = t >= window ? C.win_score[head * window + slot] : 0.f;
    dst = eviction_target(t, window, budget, P.sink, P.tau, cnt_old, z_e, C.ret_score + head * budget,
                          C.ret_pos + head * budget, red64, &slot_lds);
    cnt = cnt_old + (dst == cnt_old ? 1 : 0);
    // the share that ends the slot space always gets here: it hands the decision to the finishing launch
    if (split == nsplit - 1 && threadIdx.x == 0) ws_dst[head] = dst;
  }
  const T* k_evicted = kw + (int64_t)slot * D;  // old ring row that moves to compact slot dst
  const T* v_evicted = vw + (int64_t)slot * D;

  constexpr int RIF = GT >= 4 ? 2 : kRowsInFlight;   // rows in flight per lane group (registers: GT states per lane)
  for (int g0 = 0; g0 < G; g0 += GT) {
    float qf[GT][EPL];
    float m_run[GT], l_run[GT], acc[GT][EPL];
#pragma unroll
    for (int g = 0; g < GT; ++g) {
      Piece<T>::load(q + ((int64_t)b * P.Hq + h * G + g0 + g) * D + sub * EPL, qf[g]);
      m_run[g] = -INFINITY;
      l_run[g] = 0.f;
#pragma unroll
      for (int i = 0; i < EPL; ++i) { qf[g][i] *= P.scale; acc[g][i] = 0.f; }
    }

    for (int r0 = r_begin + wave * GPW + grp; r0 < r_end; r0 += GPB * RIF) {
      u32x4 kraw[RIF], vraw[RIF];
      bool live[RIF];
#pragma unroll
      for (int u = 0; u < RIF; ++u) {
        // Branch-free row selection so that all loads of the iteration are issued back to back; rows that do
        // not exist re-read the incoming token's row and are masked out of the softmax below.
        const int r = r0 + u * GPB;
        const bool in_ring = r < window;
        const int rr = r - window;
        live[u] = (r < r_end) && (in_ring ? r < n_valid : rr < cnt);
        const T* kp = in_ring ? kw + (int64_t)r * D : kr + (int64_t)rr * D;
        const T* vp = in_ring ? vw + (int64_t)r * D : vr + (int64_t)rr * D;
        const bool is_new = in_ring && r == slot;
        const bool is_moved = !in_ring && rr == dst;
        kp = is_moved ? k_evicted : kp;
        vp = is_moved ? v_evicted : vp;
        kp = (is_new || !live[u]) ? kn : kp;
        vp = (is_new || !live[u]) ? vn : vp;
        kraw[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(kp + sub * EPL));
        vraw[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(vp + sub * EPL));
      }
      float s[GT][RIF], m_new[GT];
#pragma unroll
      for (int g = 0; g < GT; ++g) m_new[g] = m_run[g];
#pragma unroll
      for (int u = 0; u < RIF; ++u) {
        float kf[EPL];
        Piece<T>::unpack(kraw[u], kf);
#pragma unroll
        for (int g = 0; g < GT; ++g) {
          float d = 0.f;
#pragma unroll
          for (int i = 0; i < EPL; ++i) d = fmaf(qf[g][i], kf[i], d);
#pragma unroll
          for (int off = LPR / 2; off > 0; off >>= 1) d += __shfl_xor(d, off, kWave);
          s[g][u] = live[u] ? d : -INFINITY;
          m_new[g] = fmaxf(m_new[g], s[g][u]);
        }
      }
      if (m_new[0] == -INFINITY) continue;  // nothing live for this lane group yet (liveness is the same for every g)
      float pr[GT][RIF];
#pragma unroll
      for (int g = 0; g < GT; ++g) {
        const float alpha = soft_exp<T>(m_run[g] - m_new[g]);
        l_run[g] *= alpha;
#pragma unroll
        for (int i = 0; i < EPL; ++i) acc[g][i] *= alpha;
#pragma unroll
        for (int u = 0; u < RIF; ++u) {
          pr[g][u] = soft_exp<T>(s[g][u] - m_new[g]);
          l_run[g] += pr[g][u];
        }
        m_run[g] = m_new[g];
      }
#pragma unroll
      for (int u = 0; u < RIF; ++u) {
        float vf[EPL];
        Piece<T>::unpack(vraw[u], vf);
#pragma unroll
        for (int g = 0; g < GT; ++g)
#pragma unroll
          for (int i = 0; i < EPL; ++i) acc[g][i] = fmaf(pr[g][u], vf[i], acc[g][i]);
      }
    }

    // merge the row groups of the block (fixed order -> deterministic), one query head after the other
#pragma unroll
    for (int g = 0; g < GT; ++g) {
      const int hq = h * G + g0 + g;
      if (sub == 0) { red_m[wave][grp] = m_run[g]; red_l[wave][grp] = l_run[g]; }
#pragma unroll
      for (int i = 0; i < EPL; ++i) red_acc[wave][grp][sub * EPL + i] = acc[g][i];
      __syncthreads();
      if (threadIdx.x < D) {
        float M = -INFINITY;
        for (int w = 0; w < kWaves; ++w)
          for (int gg = 0; gg < GPW; ++gg) M = fmaxf(M, red_m[w][gg]);
        float L = 0.f, A = 0.f;
        if (M != -INFINITY) {
          for (int w = 0; w < kWaves; ++w)
            for (int gg = 0; gg < GPW; ++gg) {
              const float f = soft_exp<T>(red_m[w][gg] - M);
              L = fmaf(red_l[w][gg], f, L);
              A = fmaf(red_acc[w][gg][threadIdx.x], f, A);
            }
        }
        float* rec = partial + (((int64_t)b * P.Hq + hq) * nsplit + split) * (D + 2);
        if (threadIdx.x == 0) { rec[0] = M; rec[1] = L; }
        rec[2 + threadIdx.x] = A;
      }
      __syncthreads();
    }
  }
}

template <typename T, int D>
__global__ void __launch_bounds__(kThreads)
decode_finish_kernel(CacheDev C, StepParams P, const T* __restrict__ k_new, const T* __restrict__ v_new,
                     const float* __restrict__ partial, const float* __restrict__ ws_logit,
                     const int32_t* __restrict__ ws_t, const int32_t* __restrict__ ws_dst, T* __restrict__ out) {
  const int Hkv = P.Hkv, window = P.window, budget = P.budget, rho = P.rho;
  const int b = blockIdx.x / Hkv, h = blockIdx.x - b * Hkv;
  const int64_t head = (int64_t)b * Hkv + h;
  const int tid = threadIdx.x;
  // t comes from the workspace copy made by the previous kernel: n_seen[b] itself is advanced below by the
  // h == 0 workgroup while other workgroups of the same sequence may still be starting.
  const int t = ws_t[b];
  const int slot = t % window;
  // Everything that does not depend on the eviction decision is requested first, so that the loads of the
  // decision, of the split partials and of the two rows that move are all in flight together.
  T* kw = static_cast<T*>(C.k_win) + (head * window + slot) * D;
  T* vw = static_cast<T*>(C.v_win) + (head * window + slot) * D;
  constexpr int pieces = D * (int)sizeof(T) / 16;
  const bool moves_k = tid < pieces, moves_v = tid >= pieces && tid < 2 * pieces;
  const int pc = moves_k ? tid : (moves_v ? tid - pieces : 0);
  u32x4 old_piece = {0u, 0u, 0u, 0u}, new_piece = {0u, 0u, 0u, 0u};
  if (moves_k || moves_v) {
    old_piece = reinterpret_cast<const u32x4*>(moves_k ? kw : vw)[pc];
    new_piece = reinterpret_cast<const u32x4*>((moves_k ? k_new : v_new) + head * D)[pc];
  }
  const int cnt_old = budget > 0 ? C.ret_count[head] : 0;
  const float z_e = t >= window ? C.win_score[head * window + slot] : 0.f;
  // the finalised logit of position t - rho: parked by the main launch's scoring role, or picked out of the
  // sequence's scored window (its first row is position max(0, t - 2*rho))
  float z_new = 0.f;
  if (!P.lazy && t - rho >= 0) {
    const int first = t - 2 * rho > 0 ? t - 2 * rho : 0;
    z_new = P.pre_logits != nullptr
                ? P.pre_logits[(int64_t)h * P.pre_total + (int64_t)b * P.pre_stride + (t - rho - first)]
                : ws_logit[head];
  }
  // lazy mode: the token leaving the window must have been scored by a batched scoring call
  const bool late = P.lazy && t >= window && C.n_scored[b] <= t - window;

  // ---- merge split partials of the group's query heads ------------------------------------------------------
  const int G = P.Hq / Hkv, nsplit = P.nsplit;
  for (int item = tid; item < G * D; item += kThreads) {
    const int g = item / D, d = item - g * D;
    const int64_t bh = (int64_t)b * P.Hq + h * G + g;
    const float* rec = partial + bh * nsplit * (D + 2);
    float M = -INFINITY;
    for (int s = 0; s < nsplit; ++s) M = fmaxf(M, rec[s * (D + 2)]);
    float L = 0.f, A = 0.f;
    for (int s = 0; s < nsplit; ++s) {
      const float m = rec[s * (D + 2)];
      if (m == -INFINITY) continue;
      const float f = soft_exp<T>(m - M);
      L = fmaf(rec[s * (D + 2) + 1], f, L);
      A = fmaf(rec[s * (D + 2) + 2 + d], f, A);
    }
    out[bh * D + d] = from_f32<T>(late ? __builtin_nanf("") : A / L);
  }

  __syncthreads();  // every thread holds z_e and the old ring row before anything of this head is overwritten
  // where the token leaving the window goes: decided by the main launch from the same state (eviction_target)
  const int dst = budget > 0 ? ws_dst[head] : -1;

  // ---- cache update: evicted row -> compact slot dst, then token t -> ring slot ------------------------------
  if (dst >= 0) {
    T* kr = static_cast<T*>(C.k_ret) + (head * budget + dst) * D;
    T* vr = static_cast<T*>(C.v_ret) + (head * budget + dst) * D;
    if (moves_k || moves_v) reinterpret_cast<u32x4*>(moves_k ? kr : vr)[pc] = old_piece;
    if (tid == 0) {
      const int e_pos = t - window;
      C.ret_score[head * budget + dst] = select_key(z_e, e_pos, P.sink);
      C.ret_pos[head * budget + dst] = e_pos;
      if (dst == cnt_old) C.ret_count[head] = cnt_old + 1;
    }
  }
  if (moves_k || moves_v) reinterpret_cast<u32x4*>(moves_k ? kw : vw)[pc] = new_piece;
  if (tid == 0) {
    if (!P.lazy && t - rho >= 0) C.win_score[head * window + ((t - rho) % window)] = z_new;
    if (h == 0) {
      C.n_seen[b] = t + 1;
      if (!P.lazy) C.n_scored[b] = t + 1 > rho ? t + 1 - rho : 0;
      if (late && P.status != nullptr) atomicOr(P.status, LTEA_LATE_SCORING);
    }
  }
}

size_t partial_floats(const ltea_cfg& cfg, int n_seqs, int nsplit) {
  return (size_t)n_seqs * cfg.Hq * nsplit * (cfg.D + 2);
}

int lds_row_floats(const ltea_cfg& cfg, const ltea_cnn& cnn) {
  int row_floats = 2 * cfg.D;
  for (int l = 0; l < cnn.n_layers; ++l) row_floats = cnn.c_out[l] > row_floats ? cnn.c_out[l] : row_floats;
  return row_floats;
}

struct PreScore {            // buffers of the window-scoring path, carved from the tail of the workspace
  void* win_k; void* win_v; int32_t* cu2; float* logits; void* score_ws; int64_t total;
  uint8_t* row_valid;        // windows mode only
  int stride;                // rows per sequence
};

size_t up256(size_t x) { return (x + 255) / 256 * 256; }

size_t base_workspace(const ltea_cfg& cfg, int n_seqs) {
  // sized for the larger of the two split counts
  return (partial_floats(cfg, n_seqs, decode_num_splits(cfg, n_seqs, true)) + (size_t)n_seqs * cfg.Hkv) * sizeof(float) +
         ((size_t)n_seqs + (size_t)n_seqs * cfg.Hkv) * sizeof(int32_t);
}

bool window_scoring(const ltea_cfg& cfg, const ltea_cnn& cnn) {
  return cfg.dtype == LTEA_BF16 && cnn.n_layers >= 2 && score_deep_supported(cfg, cnn);
}

// Rows per sequence of the packed windows: the receptive field, and where the register-stationary kernel scores them
// (windows mode: all windows of the batch as one sequence) as many rows of zeros as the widest dilation reaches, so that
// no tap crosses from one window into the next.
int prescore_stride(const ltea_cfg& cfg, const ltea_cnn& cnn, bool* windows_mode) {
  const int R = 2 * cnn_rho(&cnn) + 1;
  const bool wm = score_deep_reg_supported(cfg, cnn);
  if (windows_mode) *windows_mode = wm;
  if (!wm) return R;
  int gap = 0;
  for (int l = 0; l < cnn.n_layers; ++l) gap = cnn.dilation[l] > gap ? cnn.dilation[l] : gap;
  return R + gap;
}

size_t prescore_bytes(const ltea_cfg& cfg, const ltea_cnn& cnn, int n_seqs, char* base, PreScore* out) {
  bool wm = false;
  const int R = prescore_stride(cfg, cnn, &wm);
  const size_t rows = (size_t)n_seqs * R;
  uintptr_t p = reinterpret_cast<uintptr_t>(base);   // integer arithmetic: a size query carves from a null base
  auto take = [&](size_t bytes) { char* r = reinterpret_cast<char*>(p); p += up256(bytes); return r; };
  void* wk = take(rows * cfg.Hkv * cfg.D * 2);
  void* wv = take(rows * cfg.Hkv * cfg.D * 2);
  int32_t* cu2 = reinterpret_cast<int32_t*>(take(sizeof(int32_t) * (2 * (size_t)n_seqs + 1)));
  float* lg = reinterpret_cast<float*>(take(sizeof(float) * rows * cfg.Hkv));
  void* sws = take(score_deep_workspace(cfg, cnn));
  uint8_t* rv = wm ? reinterpret_cast<uint8_t*>(take(rows)) : nullptr;
  if (out) {
    out->win_k = wk; out->win_v = wv; out->cu2 = cu2; out->logits = lg; out->score_ws = sws; out->total = (int64_t)rows;
    out->row_valid = rv; out->stride = R;
  }
  return (size_t)(p - reinterpret_cast<uintptr_t>(base));
}

// cnn_or_null == nullptr selects the lazy step (no scoring; `status` receives LTEA_LATE_SCORING).
template <typename T, int D>
hipError_t run(const ltea_cfg& cfg, const ltea_cnn* cnn_or_null, const void* q, const void* k, const void* v, void* out,
               const ltea_cache& c, int n_seqs, void* workspace, bool prescore, int32_t* status, hipStream_t stream,
               const float* given_logits = nullptr, int64_t given_total = 0) {
  const bool lazy = cnn_or_null == nullptr;
  ltea_cnn none;
  memset(&none, 0, sizeof(none));
  const ltea_cnn& cnn = lazy ? none : *cnn_or_null;
  CnnDev cd;
  cd.n_layers = cnn.n_layers;
  for (int l = 0; l < LTEA_MAX_CNN_LAYERS; ++l) {
    const bool on = l < cnn.n_layers;
    cd.kernel[l] = on ? cnn.kernel[l] : 1;
    cd.dilation[l] = on ? cnn.dilation[l] : 1;
    cd.c_out[l] = on ? cnn.c_out[l] : 0;
    cd.w[l] = on ? cnn.w[l] : nullptr;
    cd.bias[l] = on ? cnn.bias[l] : nullptr;
  }
  cd.w_out = cnn.w_out;
  cd.b_out = cnn.b_out;
  CacheDev C{c.k_win, c.v_win, c.win_score, c.k_ret, c.v_ret, c.ret_score, c.ret_pos, c.ret_count, c.n_seen, c.n_scored};
  StepParams P;
  P.B = n_seqs; P.Hq = cfg.Hq; P.Hkv = cfg.Hkv; P.D = cfg.D; P.window = cfg.window; P.budget = cfg.budget;
  P.sink = cfg.sink;
  P.rho = cnn_rho(&cnn);
  P.lds_row_floats = lds_row_floats(cfg, cnn);
  P.tau = cfg.tau_logit;
  P.scale = cfg.softmax_scale > 0.f ? cfg.softmax_scale : 1.0f / sqrtf((float)cfg.D);
  const unsigned heads = (unsigned)n_seqs * (unsigned)cfg.Hkv;
  const int ks0 = cnn.kernel[0];
  P.score_mfma = (!lazy && cfg.dtype == LTEA_BF16 && cnn.n_layers == 1 && cnn.c_out[0] <= 32 && (ks0 == 3 || ks0 == 5 || ks0 == 7)) ? ks0 : 0;
  P.n_score_blocks = P.score_mfma ? cfg.Hkv * ((n_seqs + 63) / 64) : (int)heads;
  size_t lds_bytes = P.score_mfma ? 0 : (size_t)2 * (2 * P.rho + 1) * P.lds_row_floats * sizeof(float);
  P.pre_logits = nullptr;
  P.pre_total = 0;
  P.pre_stride = 2 * P.rho + 1;
  P.lazy = lazy ? 1 : 0;
  P.status = status;
  if (lazy) {
    P.n_score_blocks = (n_seqs + kThreads - 1) / kThreads;
    lds_bytes = 0;
  }
  P.pk_k = nullptr; P.pk_v = nullptr; P.pk_cu2 = nullptr; P.pk_row_valid = nullptr; P.n_pack_blocks = 0;
  PreScore ps;
  memset(&ps, 0, sizeof(ps));
  if constexpr (sizeof(T) == 2) {
    if (prescore) {
      // multi-layer bf16 CNN: the main launch packs the receptive-field windows next to its streaming (one more
      // workgroup per sequence), the fused prefill scoring kernel runs over them between the two launches of the step
      // (weights staged once per workgroup instead of once per (sequence, head)), and the finishing launch picks the
      // centre logits
      prescore_bytes(cfg, cnn, n_seqs, static_cast<char*>(workspace) + up256(base_workspace(cfg, n_seqs)), &ps);
      P.pk_k = ps.win_k; P.pk_v = ps.win_v; P.pk_cu2 = ps.cu2; P.pk_row_valid = ps.row_valid;
      P.n_pack_blocks = n_seqs;
      P.pre_logits = ps.logits;
      P.pre_total = ps.total;
      P.pre_stride = ps.stride;
      P.n_score_blocks = (n_seqs + kThreads - 1) / kThreads;
      lds_bytes = 0;
    }
  }
  P.nsplit = decode_num_splits(cfg, n_seqs, !lazy && P.pre_logits == nullptr && given_logits == nullptr);
  if (given_logits != nullptr) {   // the caller has scored the windows already (rotary models): only pick the logits
    P.pre_logits = given_logits;
    P.pre_total = given_total;
    P.n_score_blocks = (n_seqs + kThreads - 1) / kThreads;
    lds_bytes = 0;
  }
  float* partial = static_cast<float*>(workspace);
  float* ws_logit = partial + partial_floats(cfg, n_seqs, P.nsplit);
  int32_t* ws_t = reinterpret_cast<int32_t*>(ws_logit + heads);
  int32_t* ws_dst = ws_t + n_seqs;
  const unsigned grid = (unsigned)P.n_score_blocks + (unsigned)P.n_pack_blocks + heads * (unsigned)P.nsplit;
  const int G = cfg.Hq / cfg.Hkv;
  auto launch_main = [&](auto gt, auto sk) {
    hipLaunchKernelGGL((decode_main_kernel<T, D, decltype(gt)::value, decltype(sk)::value>), dim3(grid), dim3(kThreads),
                       lds_bytes, stream, cd, C, P, static_cast<const T*>(q), static_cast<const T*>(k),
                       static_cast<const T*>(v), partial, ws_logit, ws_t, ws_dst);
  };
  auto launch_gt = [&](auto sk) {
    if (G % 4 == 0) launch_main(std::integral_constant<int, 4>{}, sk);
    else if (G % 2 == 0) launch_main(std::integral_constant<int, 2>{}, sk);
    else launch_main(std::integral_constant<int, 1>{}, sk);
  };
  const int sk_run = (P.pre_logits == nullptr && !lazy) ? P.score_mfma : 0;
  if constexpr (sizeof(T) == 2) {
    if (sk_run == 3) launch_gt(std::integral_constant<int, 3>{});
    else if (sk_run == 5) launch_gt(std::integral_constant<int, 5>{});
    else if (sk_run == 7) launch_gt(std::integral_constant<int, 7>{});
    else launch_gt(std::integral_constant<int, 0>{});
  } else {
    launch_gt(std::integral_constant<int, 0>{});
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (P.n_pack_blocks > 0) {
    // windows mode: the whole batch is one sequence of n_seqs * stride rows; else two sequences per window
    const SeqView sv = ps.row_valid ? SeqView{ps.cu2, 1, ps.total, (int32_t)ps.total}
                                    : SeqView{ps.cu2, 2 * n_seqs, ps.total, 2 * P.rho + 1};
    e = launch_score_deep(cfg, cnn, ps.win_k, ps.win_v, (int64_t)cfg.Hkv * cfg.D, cfg.D, sv, ps.logits, ps.score_ws, stream,
                          ps.row_valid);
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL((decode_finish_kernel<T, D>), dim3(heads), dim3(kThreads), 0, stream, C, P,
                     static_cast<const T*>(k), static_cast<const T*>(v), partial, ws_logit, ws_t, ws_dst, static_cast<T*>(out));
  return hipGetLastError();
}

}  // namespace

// Shares of a head's rows (one workgroup each).  Measured on MI355X: when the scoring runs inside the main launch
// (single-layer bf16 CNN: a few long-running scoring workgroups) about 4096 streaming workgroups hide it best; when
// the launch only streams (lazy steps, scores computed beforehand) about 1024 fat workgroups are faster, because the
// per-workgroup prologue (eviction decision, query loads) and epilogue (cross-wave merge) then weigh less:
// decode_bf16 lazy 136 -> 129 us/step, paper stack B=32 lazy 43 -> 29 us/step, B=128 lazy 90 -> 67 us/step.
int decode_num_splits(const ltea_cfg& cfg, int n_seqs, bool scoring_inside) {
  const long heads = (long)n_seqs * cfg.Hkv;
  const int rows = cfg.window + cfg.budget;
  const long target = scoring_inside ? 4096 : 1024;
  int by_fill = (int)((target + heads - 1) / (heads > 0 ? heads : 1));
  int by_rows = (rows + 127) / 128;                                   // at least 128 rows per split
  int n = by_fill < by_rows ? by_fill : by_rows;
  if (n < 1) n = 1;
  if (n > 64) n = 64;
  return n;
}

size_t decode_workspace(const ltea_cfg& cfg, int n_seqs) { return base_workspace(cfg, n_seqs); }

// Workspace that also enables the window-scoring path of multi-layer bf16 CNNs (equal to decode_workspace otherwise).
size_t decode_workspace_full(const ltea_cfg& cfg, const ltea_cnn& cnn, int n_seqs) {
  size_t b = up256(base_workspace(cfg, n_seqs));
  if (window_scoring(cfg, cnn)) b += prescore_bytes(cfg, cnn, n_seqs, nullptr, nullptr);
  return b;
}

hipError_t launch_decode_step(const ltea_cfg& cfg, const ltea_cnn& cnn, const void* q, const void* k, const void* v,
                              void* out, const ltea_cache& c, int n_seqs, void* workspace, size_t workspace_bytes,
                              hipStream_t stream) {
  if (n_seqs == 0) return hipSuccess;
  if (cfg.dtype == LTEA_F32) {
    return cfg.D == 64 ? run<float, 64>(cfg, &cnn, q, k, v, out, c, n_seqs, workspace, false, nullptr, stream)
                       : run<float, 128>(cfg, &cnn, q, k, v, out, c, n_seqs, workspace, false, nullptr, stream);
  }
  // the window-scoring path needs the larger workspace; with the basic one the per-head path runs
  const bool prescore = window_scoring(cfg, cnn) && workspace_bytes >= decode_workspace_full(cfg, cnn, n_seqs);
  return cfg.D == 64 ? run<bf16_t, 64>(cfg, &cnn, q, k, v, out, c, n_seqs, workspace, prescore, nullptr, stream)
                     : run<bf16_t, 128>(cfg, &cnn, q, k, v, out, c, n_seqs, workspace, prescore, nullptr, stream);
}

size_t decode_windows_layout(const ltea_cfg& cfg, int rho, int n_seqs, void* base, DecodeWindows* out) {
  const size_t esz = cfg.dtype == LTEA_F32 ? 4 : 2;
  const size_t rows = (size_t)n_seqs * (2 * rho + 1);
  uintptr_t p = reinterpret_cast<uintptr_t>(base);
  auto take = [&](size_t bytes) { char* r = reinterpret_cast<char*>(p); p += up256(bytes); return r; };
  void* wk = take(rows * cfg.Hkv * cfg.D * esz);
  void* wv = take(rows * cfg.Hkv * cfg.D * esz);
  int32_t* cu2 = reinterpret_cast<int32_t*>(take(sizeof(int32_t) * (2 * (size_t)n_seqs + 1)));
  float* lg = reinterpret_cast<float*>(take(sizeof(float) * rows * cfg.Hkv));
  if (out) { out->win_k = wk; out->win_v = wv; out->cu2 = cu2; out->logits = lg; out->total = (int64_t)rows; }
  return (size_t)(p - reinterpret_cast<uintptr_t>(base));
}

hipError_t launch_decode_windows(const ltea_cfg& cfg, int rho, const void* k, const void* v, const void* k_feat,
                                 const ltea_rope* rope, int32_t* status, const ltea_cache& c, int n_seqs,
                                 const DecodeWindows& w, hipStream_t stream) {
  CacheDev C{c.k_win, c.v_win, c.win_score, c.k_ret, c.v_ret, c.ret_score, c.ret_pos, c.ret_count, c.n_seen, c.n_scored};
  auto go = [&](auto tag) {
    using T = decltype(tag);
    hipLaunchKernelGGL(decode_windows_kernel<T>, dim3((unsigned)n_seqs), dim3(256), 0, stream, C,
                       static_cast<const T*>(k), static_cast<const T*>(v), static_cast<const T*>(k_feat), rope_dev(rope),
                       status, static_cast<T*>(w.win_k), static_cast<T*>(w.win_v), w.cu2, n_seqs, cfg.Hkv, cfg.D,
                       cfg.window, rho, 2 * rho + 1, static_cast<uint8_t*>(nullptr));
  };
  if (cfg.dtype == LTEA_F32) go(float{});
  else go(bf16_t{});
  return hipGetLastError();
}

hipError_t launch_decode_step_scored(const ltea_cfg& cfg, const ltea_cnn& cnn, const void* q, const void* k,
                                     const void* v, void* out, const ltea_cache& c, int n_seqs, void* workspace,
                                     const float* logits, int64_t logits_total, hipStream_t stream) {
  if (n_seqs == 0) return hipSuccess;
  if (cfg.dtype == LTEA_F32) {
    return cfg.D == 64 ? run<float, 64>(cfg, &cnn, q, k, v, out, c, n_seqs, workspace, false, nullptr, stream, logits, logits_total)
                       : run<float, 128>(cfg, &cnn, q, k, v, out, c, n_seqs, workspace, false, nullptr, stream, logits, logits_total);
  }
  return cfg.D == 64 ? run<bf16_t, 64>(cfg, &cnn, q, k, v, out, c, n_seqs, workspace, false, nullptr, stream, logits, logits_total)
                     : run<bf16_t, 128>(cfg, &cnn, q, k, v, out, c, n_seqs, workspace, false, nullptr, stream, logits, logits_total);
}

hipError_t launch_decode_step_lazy(const ltea_cfg& cfg, const void* q, const void* k, const void* v, void* out,
                                   const ltea_cache& c, int n_seqs, int32_t* status, void* workspace,
                                   hipStream_t stream) {
  if (n_seqs == 0) return hipSuccess;
  if (cfg.dtype == LTEA_F32) {
    return cfg.D == 64 ? run<float, 64>(cfg, nullptr, q, k, v, out, c, n_seqs, workspace, false, status, stream)
                       : run<float, 128>(cfg, nullptr, q, k, v, out, c, n_seqs, workspace, false, status, stream);
  }
  return cfg.D == 64 ? run<bf16_t, 64>(cfg, nullptr, q, k, v, out, c, n_seqs, workspace, false, status, stream)
                     : run<bf16_t, 128>(cfg, nullptr, q, k, v, out, c, n_seqs, workspace, false, status, stream);
}

}  // namespace ltea
