// Backward of the scoring CNN of the LTE module (paper Section 3.1.1; trained through the gradient of the logits
// that Section 3.1.2 defines): from d(loss)/d(logit) to the gradients of every conv weight, bias, the output
// projection and the input features.  fp32-accurate arithmetic for any depth and either storage type, as LDS-tiled
// products on the fp32 matrix instruction, or, on bf16 storage where one operand is a bf16 value, on the bf16 one with
// the fp32 operand split into three bf16 terms.  The module is small next to the attention (paper stack: 65 kflop
// per token-head forward).  Everything is summed in a fixed order: same bits every run.
//
//   1. forward again, keeping the pre-activations y_l and the activations a_l = silu(y_l) of every layer
//      (fp32 [Hkv][T][C_l] each); the features of layer 0 are copied to a dense fp32 array first unless the bf16
//      kernels read k / v themselves;
//   2. d y_L = dz * w_out * silu'(y_L);  d w_out = sum_t dz * silu(y_L),  d b_out = sum_t dz;
//   3. for l = L .. 1:  d bias_l = sum_t d y_l;
//                       d W_l[c][m][tap] = sum_t d y_l[t][c] * a_{l-1}[t + off(tap)][m]      (inside the sequence)
//                       d a_{l-1}[t][m]  = sum_{tap, c} W_l[c][m][tap] * d y_l[t - off(tap)][c]
//                       d y_{l-1} = d a_{l-1} * silu'(y_{l-1})        (l > 1)   or   dk, dv = d a_0   (l = 1).
// Sums over tokens are taken in two stages: per chunk of kTokChunk (weights) or kColChunk (column sums) tokens into a
// partial array, then over the chunks.
#include <type_traits>

#include "ltea_common.h"
#include "ltea_kernels.h"
#include "rope_dev.h"
#include "mfma_tiles.h"

namespace ltea {
namespace {

constexpr int kTokChunk = 512;   // tokens per partial of the weight products
constexpr int kColChunk = 128;   // tokens per partial of the column sums

__device__ __forceinline__ float silu_grad_f32(float y) {
  const float s = 1.0f / (1.0f + expf(-y));
  return s * (1.0f + y * (1.0f - s));
}

// seq_lo[t], seq_hi[t]: bounds of the sequence token t belongs to.
__global__ void __launch_bounds__(256)
token_bounds_kernel(const int32_t* __restrict__ cu, int n_seqs, int64_t total, int32_t* __restrict__ seq_lo,
                    int32_t* __restrict__ seq_hi) {
  const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (t >= total) return;
  const int s = find_sequence(cu, n_seqs, t);
  seq_lo[t] = cu[s];
  seq_hi[t] = cu[s + 1];
}

// d y_L[h][t][c] = dz[h][t] * w_out[h][c] * silu'(y_L[h][t][c])
template <typename T>
__global__ void __launch_bounds__(256)
out_proj_backward_kernel(const float* __restrict__ dz, const T* __restrict__ w_out, const float* __restrict__ pre, int C,
                         int64_t total, float* __restrict__ dpre) {
  const int h = blockIdx.y;
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t tok = idx / C;
  const int c = (int)(idx - tok * C);
  if (tok >= total) return;
  const int64_t i = ((int64_t)h * total + tok) * C + c;
  dpre[i] = dz[(int64_t)h * total + tok] * to_f32(w_out[(int64_t)h * C + c]) * silu_grad_f32(pre[i]);
}

// Layer-0 input as a dense fp32 array: a0[h][t][m] = concat(key, value) features of token t, moved in 16-byte pieces of
// the storage type (rows of D elements are whole pieces).
template <typename T>
__global__ void __launch_bounds__(256)
features_kernel(const T* __restrict__ k, const T* __restrict__ v, int64_t stride_tok, int64_t stride_head, int D,
                int64_t total, float* __restrict__ a0) {
  constexpr int EPP = Elems<T>::N;
  const int h = blockIdx.y;
  const int pieces = 2 * D / EPP;
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t tok = idx / pieces;
  const int m = (int)(idx - tok * pieces) * EPP;
  if (tok >= total) return;
  const T* src = (m < D ? k : v) + tok * stride_tok + (int64_t)h * stride_head + (m < D ? m : m - D);
  float x[EPP];
  Elems<T>::unpack(*reinterpret_cast<const u32x4*>(src), x);
  float4* dst = reinterpret_cast<float4*>(a0 + ((int64_t)h * total + tok) * 2 * D + m);
#pragma unroll
  for (int i = 0; i < EPP / 4; ++i) dst[i] = make_float4(x[4 * i], x[4 * i + 1], x[4 * i + 2], x[4 * i + 3]);
}

// The weights of one layer as two fp32 panels per head: wf[h][tap][m][c] (contraction over the input channels m: the
// forward) and wb[h][tap][c][m] (contraction over the output channels c: the backward towards the input);
// wq and wqf, when given, are wb's and wf's order in the storage type (operands of the bf16 matrix instruction on
// bf16 storage: the first layer's forward, and the products towards the input).
template <typename T>
__global__ void __launch_bounds__(256)
weight_panels_kernel(const T* __restrict__ W, int Cin, int Cout, int ks, int64_t n, float* __restrict__ wf,
                     float* __restrict__ wb, T* __restrict__ wq, T* __restrict__ wqf) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;     // over [h][c][m][tap]
  if (i >= n) return;
  const int tap = (int)(i % ks);
  const int m = (int)((i / ks) % Cin);
  const int c = (int)((i / ((int64_t)ks * Cin)) % Cout);
  const int64_t h = i / ((int64_t)ks * Cin * Cout);
  const float w = to_f32(W[i]);
  wf[((h * ks + tap) * Cin + m) * Cout + c] = w;
  wb[((h * ks + tap) * Cout + c) * Cin + m] = w;
  if (wq != nullptr) wq[((h * ks + tap) * Cout + c) * Cin + m] = W[i];     // wb's order in the storage type
  if (wqf != nullptr) wqf[((h * ks + tap) * Cin + m) * Cout + c] = W[i];   // wf's order in the storage type
}

// The fp32 products below run on v_mfma_f32_32x32x2_f32 (fp32 operands, two contraction steps per instruction: lane l
// supplies row / column l % 32 of step l / 32), their operands staged through LDS.  Weight products: up to TM input
// channels x TN output channels per workgroup in 32 x 32 pieces per wave; conv products: TN outputs wide.
constexpr int TM = 64, TN = 64;
// conv products: TMC tokens per workgroup (two 32-token sub-tiles per wave), contraction slices of KCC channels, up
// to GT taps per stage whose rows reach at most HALO past the tile; LDS row strides RSA / RSB keep the 16-byte operand
// reads of 16 neighbouring lanes, and the two lane halves' weight reads, on different banks
constexpr int TMC = 128, KCC = 16, HALO = 64, GT = 3, RSA = KCC + 4, RSB = 72;
constexpr int A_ROWS = TMC + HALO, PA = A_ROWS * (KCC / 4) / 256, PB = GT * KCC * (TN / 4) / 256;
static_assert(A_ROWS * (KCC / 4) % 256 == 0 && GT * KCC * (TN / 4) % 256 == 0, "whole quads per thread");
constexpr int KCW = 32, PERW = KCW * TM / 256;   // weight products: tokens per contraction slice

// row[x .. x+3] of a readable row of `limit` floats, loaded unconditionally from addresses clamped into the row, with
// a 4-bit mask of the elements that count (those below the limit, none when !ok).  The caller zeroes the others where
// it consumes the quad, so that a thread's loads of a stage are all in flight together and none is waited for before
// then.  VEC: limit % 4 == 0 and the row starts on a 16-byte boundary, so a quad is inside or outside as a whole.
template <bool VEC>
__device__ __forceinline__ float4 load_quad(const float* __restrict__ row, int x, int limit, bool ok, unsigned& mask4) {
  if constexpr (VEC) {
    mask4 = (ok && x < limit) ? 0xFu : 0u;
    return *reinterpret_cast<const float4*>(row + min(x, limit - 4));
  } else {
    const int last = limit - 1;
    mask4 = 0u;
#pragma unroll
    for (int c = 0; c < 4; ++c) mask4 |= (ok && x + c < limit) ? 1u << c : 0u;
    return make_float4(row[min(x, last)], row[min(x + 1, last)], row[min(x + 2, last)], row[min(x + 3, last)]);
  }
}

// v if keep, else zero.  The empty asm makes the loaded value needed either way, so the load stays where it was issued
// instead of moving under a condition (and being waited for at once).
__device__ __forceinline__ float masked_value(float v, bool keep) {
  asm volatile("" : "+v"(v));
  return keep ? v : 0.f;
}

// The quad with the elements outside the mask zeroed.  The empty asm makes the loaded value needed whatever the mask
// says, so the load stays where it was issued instead of moving under a condition.
__device__ __forceinline__ float4 masked_quad(float4 v, unsigned mask4) {
  asm volatile("" : "+v"(v.x), "+v"(v.y), "+v"(v.z), "+v"(v.w));
  return make_float4(mask4 & 1u ? v.x : 0.f, mask4 & 2u ? v.y : 0.f, mask4 & 4u ? v.z : 0.f, mask4 & 8u ? v.w : 0.f);
}

// out[t][n] = sum_tap sum_k in[t + sign * off(tap)][k] * wt[tap][k][n]   (rows outside t's sequence count as zero)
// for one head, as a tiled fp32 product: TMC tokens x TN outputs per workgroup.  A stage brings one contraction slice
// of KCC channels into LDS: the input rows of the tile plus the extra rows that a group of up to GT taps reaches
// (at most HALO), and those taps' weight rows; every staged input row then serves all taps of the group.  Whether a
// tap's row lies in the token's own sequence is decided where the operand is read.  What is done with the result:
//   mode 0 (forward)          pre = out + bias, act = silu(pre)
//   mode 1 (hidden backward)  dpre_out = out * silu'(pre_prev)
//   mode 2 (input backward)   dk / dv [T][Hkv][D] of the storage type (n < D: key part)
template <typename T, bool VEC, bool NARROW>
__global__ void __launch_bounds__(256, 4)
conv_product_kernel(const float* __restrict__ in, const float* __restrict__ wt, int K, int N, int ks, int dil, int sign,
                    const int32_t* __restrict__ seq_lo, const int32_t* __restrict__ seq_hi, int64_t total, int Hkv,
                    int mode, const float* __restrict__ bias, const float* __restrict__ pre_prev,
                    float* __restrict__ out0, float* __restrict__ out1, T* __restrict__ dk, T* __restrict__ dv, int D) {
  __shared__ __align__(16) float a_s[A_ROWS][RSA];     // [staged input row][channel of the slice]
  __shared__ __align__(16) float b_s[GT * KCC][RSB];   // [tap of the group][channel of the slice][output]
  const int h = blockIdx.z;
  const int64_t t0 = (int64_t)blockIdx.x * TMC;
  const int n0 = blockIdx.y * TN;
  const int tid = threadIdx.x;
  const float* in_h = in + (int64_t)h * total * K;
  const float* wt_h = wt + (int64_t)h * ks * K * N;
  const int half = (ks - 1) / 2;
  const int lane = tid & 63, wv = tid >> 6, ql = lane & 31, hb = lane >> 5;
  // Wave roles.  Wide: the waves form 2 x 2, each with two 32-token sub-tiles and one 32-column half of the outputs.
  // NARROW (N <= 32): the four waves take 32 tokens each and the one column half there is.
  constexpr int U = NARROW ? 1 : 2;
  const int row0 = NARROW ? 32 * wv : 64 * (wv >> 1), col0 = NARROW ? 0 : 32 * (wv & 1);
  // the wave's two token rows per lane, and the bounds of their sequences
  int64_t tok[U];
  int lo[U], hi[U];
#pragma unroll
  for (int u = 0; u < U; ++u) {
    tok[u] = t0 + row0 + 32 * u + ql;
    const bool ok = tok[u] < total;
    lo[u] = ok ? seq_lo[tok[u]] : 0;
    hi[u] = ok ? seq_hi[tok[u]] : 0;
  }
  f32x16 acc[U];         // wide: two token sub-tiles of 32 per wave, every weight operand read serves two MFMAs
#pragma unroll
  for (int u = 0; u < U; ++u)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[u][r] = 0.f;
  const int per_group = min(GT, 1 + HALO / dil);       // taps whose rows fit the staged halo
  const int groups = (ks + per_group - 1) / per_group;
  const int slices = (K + KCC - 1) / KCC, stages = groups * slices;
  // of a stage: first tap, number of taps, and the offset of the first staged row from the tile's first token
  auto stage_taps = [&](int stage, int& tap0, int& ntap, int& k0, int& base_off) {
    const int g = stage / slices;
    k0 = (stage - g * slices) * KCC;
    tap0 = g * per_group;
    ntap = min(per_group, ks - tap0);
    base_off = sign > 0 ? (tap0 - half) * dil : -(tap0 + ntap - 1 - half) * dil;
  };
  // The next stage's operands are fetched into registers while the current one is multiplied.
  float4 ra[PA], rb[PB];
  unsigned mask_a, mask_b;       // four bits per quad: which of its elements count
  auto fetch = [&](int stage) {
    int tap0, ntap, k0, base_off;
    stage_taps(stage, tap0, ntap, k0, base_off);
    const int rows = TMC + (ntap - 1) * dil;
    mask_a = mask_b = 0u;
#pragma unroll
    for (int i = 0; i < PA; ++i) {
      const int e = tid + 256 * i, row = e / (KCC / 4), q = e % (KCC / 4);
      const int64_t p = t0 + row + base_off;
      const bool ok = row < rows && p >= 0 && p < total;
      unsigned m4;
      ra[i] = load_quad<VEC>(in_h + (ok ? p : 0) * K, k0 + 4 * q, K, ok, m4);
      mask_a |= m4 << (4 * i);
    }
#pragma unroll
    for (int i = 0; i < PB; ++i) {
      const int e = tid + 256 * i, jrow = e / (TN / 4), q = e % (TN / 4);
      const int j = jrow / KCC, kk = jrow % KCC;
      const bool ok = j < ntap && k0 + kk < K;
      unsigned m4;
      rb[i] = load_quad<VEC>(wt_h + (ok ? ((int64_t)(tap0 + j) * K + k0 + kk) * N : 0), n0 + 4 * q, N, ok, m4);
      mask_b |= m4 << (4 * i);
    }
  };
  fetch(0);
  for (int stage = 0; stage < stages; ++stage) {
    __syncthreads();     // the previous stage's tiles are no longer read
#pragma unroll
    for (int i = 0; i < PA; ++i) {
      const int e = tid + 256 * i;
      *reinterpret_cast<float4*>(&a_s[e / (KCC / 4)][4 * (e % (KCC / 4))]) = masked_quad(ra[i], mask_a >> (4 * i));
    }
#pragma unroll
    for (int i = 0; i < PB; ++i) {
      const int e = tid + 256 * i;
      *reinterpret_cast<float4*>(&b_s[e / (TN / 4)][4 * (e % (TN / 4))]) = masked_quad(rb[i], mask_b >> (4 * i));
    }
    __syncthreads();
    int tap0, ntap, k0, base_off;
    stage_taps(stage, tap0, ntap, k0, base_off);
    if (stage + 1 < stages) fetch(stage + 1);
    const int kgroups = (min(KCC, K - k0) + 7) / 8;
    for (int j = 0; j < ntap; ++j) {
      const int off = sign * (tap0 + j - half) * dil;
      const int shift = off - base_off;                 // 0 .. (ntap-1)*dil
      bool valid[U];
#pragma unroll
      for (int u = 0; u < U; ++u) valid[u] = tok[u] + off >= lo[u] && tok[u] + off < hi[u];
      // Lane half hb takes channels 8g + 4hb .. 8g + 4hb + 3 of each group of eight, one per MFMA, from both operands.
      for (int g = 0; g < kgroups; ++g) {
        float4 a[U];
#pragma unroll
        for (int u = 0; u < U; ++u)
          a[u] = *reinterpret_cast<const float4*>(&a_s[row0 + 32 * u + ql + shift][8 * g + 4 * hb]);
        const float* bp = &b_s[j * KCC + 8 * g + 4 * hb][col0 + ql];
        const float b0 = bp[0], b1 = bp[RSB], b2 = bp[2 * RSB], b3 = bp[3 * RSB];
#pragma unroll
        for (int u = 0; u < U; ++u) a[u] = masked_quad(a[u], valid[u] ? 0xFu : 0u);
#pragma unroll
        for (int u = 0; u < U; ++u) acc[u] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[u].x, b0, acc[u], 0, 0, 0);
#pragma unroll
        for (int u = 0; u < U; ++u) acc[u] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[u].y, b1, acc[u], 0, 0, 0);
#pragma unroll
        for (int u = 0; u < U; ++u) acc[u] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[u].z, b2, acc[u], 0, 0, 0);
#pragma unroll
        for (int u = 0; u < U; ++u) acc[u] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[u].w, b3, acc[u], 0, 0, 0);
      }
    }
  }
  // accumulator register r of lane half hb: token row 8*(r/4) + 4*hb + r%4 of the sub-tile, output column ql
  const int n = n0 + col0 + ql;
  const bool n_ok = n < N;
  auto token_of = [&](int ur) { return t0 + row0 + 32 * (ur / 16) + 8 * ((ur % 16) / 4) + 4 * hb + (ur % 4); };
  if (mode == 0) {
    const float bv = n_ok ? bias[(int64_t)h * N + n] : 0.f;
#pragma unroll
    for (int ur = 0; ur < 16 * U; ++ur) {
      const int64_t t = token_of(ur);
      if (t >= total || !n_ok) continue;
      const int64_t o = ((int64_t)h * total + t) * N + n;
      const float y = acc[ur / 16][ur % 16] + bv;
      out0[o] = y;
      out1[o] = silu_f32(y);
    }
  } else if (mode == 1) {
    // per sub-tile, all of the lane's pre-activations are requested before the first is used
#pragma unroll
    for (int u = 0; u < U; ++u) {
      float pp[16];
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int64_t t = token_of(16 * u + r);
        pp[r] = pre_prev[(t < total && n_ok) ? ((int64_t)h * total + t) * N + n : 0];
      }
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int64_t t = token_of(16 * u + r);
        if (t >= total || !n_ok) continue;
        out0[((int64_t)h * total + t) * N + n] = acc[u][r] * silu_grad_f32(pp[r]);
      }
    }
  } else {
    T* dst = n < D ? dk : dv;
    const int col = n < D ? n : n - D;
    if (dst != nullptr && n_ok) {
#pragma unroll
      for (int ur = 0; ur < 16 * U; ++ur) {
        const int64_t t = token_of(ur);
        if (t < total) dst[(t * Hkv + h) * D + col] = from_f32<T>(acc[ur / 16][ur % 16]);
      }
    }
  }
}

// Forward of the first layer on bf16 storage: pre = bias + sum_tap sum_m x[t + off(tap)][m] * W[c][m][tap] with x the
// token's key and value features.  Both operands are bf16 values, so their products are exact in fp32 and the bf16
// matrix instruction (v_mfma_f32_32x32x16_bf16, fp32 accumulation) gives what the fp32 one would at 16 times the rate.
// Same tiling as conv_product_kernel: TMC tokens x TN outputs per workgroup, slices of KCB channels (a slice lies in
// the keys or in the values), the rows of a group of taps staged once; rows are read straight from k / v.
constexpr int KCB = 32, RSQ = KCB + 8;     // channels per slice; LDS row stride in elements (16-byte reads of 16 lanes
                                           // then cover all banks)
constexpr int PQA = A_ROWS * (KCB / 8) / 256, PQB = GT * TN * (KCB / 8) / 256;
static_assert(A_ROWS * (KCB / 8) % 256 == 0 && GT * TN * (KCB / 8) % 256 == 0, "whole 16-byte pieces per thread");

template <bool NARROW>
__global__ void __launch_bounds__(256, 4)
conv_first_bf16_kernel(const bf16_t* __restrict__ k, const bf16_t* __restrict__ v, int64_t stride_tok, int64_t stride_head,
                       const bf16_t* __restrict__ wq, int D, int N, int ks, int dil, const int32_t* __restrict__ seq_lo,
                       const int32_t* __restrict__ seq_hi, int64_t total, const float* __restrict__ bias,
                       float* __restrict__ pre, float* __restrict__ act) {
  __shared__ __align__(16) bf16_t a_s[A_ROWS][RSQ];       // [staged token row][channel of the slice]
  __shared__ __align__(16) bf16_t b_s[GT][TN][RSQ];       // [tap of the group][output][channel of the slice]
  const int K = 2 * D;
  const int h = blockIdx.z;
  const int64_t t0 = (int64_t)blockIdx.x * TMC;
  const int n0 = blockIdx.y * TN;
  const int tid = threadIdx.x;
  const bf16_t* w_h = wq + (int64_t)h * ks * N * K;
  const int half = (ks - 1) / 2;
  const int lane = tid & 63, wv = tid >> 6, ql = lane & 31, hb = lane >> 5;
  constexpr int U = NARROW ? 1 : 2;                       // wave roles as in conv_product_kernel
  const int row0 = NARROW ? 32 * wv : 64 * (wv >> 1), col0 = NARROW ? 0 : 32 * (wv & 1);
  int64_t tok[U];
  int lo[U], hi[U];
#pragma unroll
  for (int u = 0; u < U; ++u) {
    tok[u] = t0 + row0 + 32 * u + ql;
    const bool ok = tok[u] < total;
    lo[u] = ok ? seq_lo[tok[u]] : 0;
    hi[u] = ok ? seq_hi[tok[u]] : 0;
  }
  f32x16 acc[U];
#pragma unroll
  for (int u = 0; u < U; ++u)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[u][r] = 0.f;
  const int per_group = min(GT, 1 + HALO / dil);
  const int groups = (ks + per_group - 1) / per_group;
  const int slices = K / KCB, stages = groups * slices;   // D is a multiple of KCB
  auto stage_taps = [&](int stage, int& tap0, int& ntap, int& k0, int& base_off) {
    const int g = stage / slices;
    k0 = (stage - g * slices) * KCB;
    tap0 = g * per_group;
    ntap = min(per_group, ks - tap0);
    base_off = (tap0 - half) * dil;
  };
  u32x4 ra[PQA], rb[PQB];
  unsigned keep_a, keep_b;       // one bit per 16-byte piece: does it count
  auto fetch = [&](int stage) {
    int tap0, ntap, k0, base_off;
    stage_taps(stage, tap0, ntap, k0, base_off);
    const int rows = TMC + (ntap - 1) * dil;
    const bf16_t* src = (k0 < D ? k + k0 : v + (k0 - D)) + (int64_t)h * stride_head;
    keep_a = keep_b = 0u;
#pragma unroll
    for (int i = 0; i < PQA; ++i) {
      const int e = tid + 256 * i, row = e / (KCB / 8), q = e % (KCB / 8);
      const int64_t p = t0 + row + base_off;
      const bool ok = row < rows && p >= 0 && p < total;
      ra[i] = *reinterpret_cast<const u32x4*>(src + (ok ? p : 0) * stride_tok + 8 * q);   // unconditional, inside the array
      keep_a |= ok ? 1u << i : 0u;
    }
#pragma unroll
    for (int i = 0; i < PQB; ++i) {
      const int e = tid + 256 * i, jn = e / (KCB / 8), q = e % (KCB / 8);
      const int j = jn / TN, n = jn % TN;
      const bool ok = j < ntap && n0 + n < N;
      rb[i] = *reinterpret_cast<const u32x4*>(w_h + (ok ? ((int64_t)(tap0 + j) * N + n0 + n) * K : 0) + k0 + 8 * q);
      keep_b |= ok ? 1u << i : 0u;
    }
  };
  auto masked_piece = [](u32x4 x, bool keep) {
    asm volatile("" : "+v"(x));      // the loaded value is needed whatever the mask says: the load stays unconditional
    return keep ? x : u32x4{0u, 0u, 0u, 0u};
  };
  fetch(0);
  for (int stage = 0; stage < stages; ++stage) {
    __syncthreads();
#pragma unroll
    for (int i = 0; i < PQA; ++i) {
      const int e = tid + 256 * i;
      *reinterpret_cast<u32x4*>(&a_s[e / (KCB / 8)][8 * (e % (KCB / 8))]) = masked_piece(ra[i], keep_a >> i & 1u);
    }
#pragma unroll
    for (int i = 0; i < PQB; ++i) {
      const int e = tid + 256 * i, jn = e / (KCB / 8);
      *reinterpret_cast<u32x4*>(&b_s[jn / TN][jn % TN][8 * (e % (KCB / 8))]) = masked_piece(rb[i], keep_b >> i & 1u);
    }
    __syncthreads();
    int tap0, ntap, k0, base_off;
    stage_taps(stage, tap0, ntap, k0, base_off);
    if (stage + 1 < stages) fetch(stage + 1);
    for (int j = 0; j < ntap; ++j) {
      const int off = (tap0 + j - half) * dil;
      const int shift = off - base_off;
      bool valid[U];
#pragma unroll
      for (int u = 0; u < U; ++u) valid[u] = tok[u] + off >= lo[u] && tok[u] + off < hi[u];
      // lane half hb supplies channels 16 s + 8 hb .. + 7 of its row (tokens) / column (outputs) to step s
#pragma unroll
      for (int sk = 0; sk < KCB / 16; ++sk) {
        u32x4 a[U];
#pragma unroll
        for (int u = 0; u < U; ++u) a[u] = *reinterpret_cast<const u32x4*>(&a_s[row0 + 32 * u + ql + shift][16 * sk + 8 * hb]);
        const u32x4 b = *reinterpret_cast<const u32x4*>(&b_s[j][col0 + ql][16 * sk + 8 * hb]);
#pragma unroll
        for (int u = 0; u < U; ++u) {
          a[u] = masked_piece(a[u], valid[u]);
          acc[u] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a[u]), __builtin_bit_cast(bf16x8, b),
                                                          acc[u], 0, 0, 0);
        }
      }
    }
  }
  // accumulator register r of lane half hb: token row 8*(r/4) + 4*hb + r%4 of the sub-tile, output column ql
  const int n = n0 + col0 + ql;
  if (n >= N) return;
  const float bv = bias[(int64_t)h * N + n];
#pragma unroll
  for (int ur = 0; ur < 16 * U; ++ur) {
    const int64_t t = t0 + row0 + 32 * (ur / 16) + 8 * ((ur % 16) / 4) + 4 * hb + (ur % 4);
    if (t >= total) continue;
    const int64_t o = ((int64_t)h * total + t) * N + n;
    const float y = acc[ur / 16][ur % 16] + bv;
    pre[o] = y;
    act[o] = silu_f32(y);
  }
}

// Towards the input on bf16 storage: out[t][m] = sum_tap sum_c d y[t - off(tap)][c] * W[c][m][tap].  The weights are
// bf16 values; the fp32 d y is split into three bf16 terms (x = hi + mid + lo up to 2^-24 of x), whose products with
// the weights are exact in fp32, so three bf16 matrix instructions give the fp32 product at about five times the fp32
// instruction's rate.  Tiling as conv_product_kernel, slices of KCS channels; used when K and N are multiples of 8.
// mode 1: dpre_out = out * silu'(pre_prev);  mode 2: dk / dv [T][Hkv][D] (n < D: key part).
constexpr int KCS = 16, RSS = KCS + 8;     // channels per slice; LDS row stride in elements
constexpr int PSA = A_ROWS * (KCS / 4) / 256, PSB = (GT * TN * (KCS / 8) + 255) / 256;
static_assert(A_ROWS * (KCS / 4) % 256 == 0, "whole quads per thread");

template <bool NARROW>
__global__ void __launch_bounds__(256, 4)
conv_back_bf16_kernel(const float* __restrict__ in, const bf16_t* __restrict__ wqf, int K, int N, int ks, int dil,
                      const int32_t* __restrict__ seq_lo, const int32_t* __restrict__ seq_hi, int64_t total, int Hkv,
                      int mode, const float* __restrict__ pre_prev, float* __restrict__ out0, bf16_t* __restrict__ dk,
                      bf16_t* __restrict__ dv, int D) {
  __shared__ __align__(16) bf16_t a_s[3][A_ROWS][RSS];    // [term of the split][staged token row][channel of the slice]
  __shared__ __align__(16) bf16_t b_s[GT][TN][RSS];       // [tap of the group][output][channel of the slice]
  const int h = blockIdx.z;
  const int64_t t0 = (int64_t)blockIdx.x * TMC;
  const int n0 = blockIdx.y * TN;
  const int tid = threadIdx.x;
  const float* in_h = in + (int64_t)h * total * K;
  const bf16_t* w_h = wqf + (int64_t)h * ks * N * K;
  const int half = (ks - 1) / 2;
  const int lane = tid & 63, wv = tid >> 6, ql = lane & 31, hb = lane >> 5;
  constexpr int U = NARROW ? 1 : 2;                       // wave roles as in conv_product_kernel
  const int row0 = NARROW ? 32 * wv : 64 * (wv >> 1), col0 = NARROW ? 0 : 32 * (wv & 1);
  int64_t tok[U];
  int lo[U], hi[U];
#pragma unroll
  for (int u = 0; u < U; ++u) {
    tok[u] = t0 + row0 + 32 * u + ql;
    const bool ok = tok[u] < total;
    lo[u] = ok ? seq_lo[tok[u]] : 0;
    hi[u] = ok ? seq_hi[tok[u]] : 0;
  }
  f32x16 acc[U];
#pragma unroll
  for (int u = 0; u < U; ++u)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[u][r] = 0.f;
  const int per_group = min(GT, 1 + HALO / dil);
  const int groups = (ks + per_group - 1) / per_group;
  const int slices = (K + KCS - 1) / KCS, stages = groups * slices;
  // taps are mirrored: tap j of a group reads row t - (tap - half) * dil; the group's lowest row belongs to its last tap
  auto stage_taps = [&](int stage, int& tap0, int& ntap, int& k0, int& base_off) {
    const int g = stage / slices;
    k0 = (stage - g * slices) * KCS;
    tap0 = g * per_group;
    ntap = min(per_group, ks - tap0);
    base_off = -(tap0 + ntap - 1 - half) * dil;
  };
  float4 ra[PSA];
  u32x4 rb[PSB];
  unsigned keep_a, keep_b;
  auto fetch = [&](int stage) {
    int tap0, ntap, k0, base_off;
    stage_taps(stage, tap0, ntap, k0, base_off);
    const int rows = TMC + (ntap - 1) * dil;
    keep_a = keep_b = 0u;
#pragma unroll
    for (int i = 0; i < PSA; ++i) {
      const int e = tid + 256 * i, row = e / (KCS / 4), q = e % (KCS / 4);
      const int64_t p = t0 + row + base_off;
      const bool ok = row < rows && p >= 0 && p < total && k0 + 4 * q < K;          // K % 4 == 0: whole quads
      ra[i] = *reinterpret_cast<const float4*>(in_h + (ok ? p : 0) * K + min(k0 + 4 * q, K - 4));
      keep_a |= ok ? 1u << i : 0u;
    }
#pragma unroll
    for (int i = 0; i < PSB; ++i) {
      const int e = tid + 256 * i, jn = e / (KCS / 8), q = e % (KCS / 8);
      const int j = jn / TN, n = jn % TN;
      const bool ok = e < GT * TN * (KCS / 8) && j < ntap && n0 + n < N && k0 + 8 * q < K;   // K % 8 == 0: whole pieces
      rb[i] = *reinterpret_cast<const u32x4*>(w_h + (ok ? ((int64_t)(tap0 + j) * N + n0 + n) * K : 0) + min(k0 + 8 * q, K - 8));
      keep_b |= ok ? 1u << i : 0u;
    }
  };
  auto masked_piece = [](u32x4 x, bool keep) {
    asm volatile("" : "+v"(x));      // the loaded value is needed whatever the mask says: the load stays unconditional
    return keep ? x : u32x4{0u, 0u, 0u, 0u};
  };
  auto bits = [](float x) { return (uint32_t)__builtin_bit_cast(uint16_t, from_f32<bf16_t>(x)); };
  fetch(0);
  for (int stage = 0; stage < stages; ++stage) {
    __syncthreads();
#pragma unroll
    for (int i = 0; i < PSA; ++i) {
      const int e = tid + 256 * i, row = e / (KCS / 4), q = e % (KCS / 4);
      const float4 x = masked_quad(ra[i], (keep_a >> i & 1u) ? 0xFu : 0u);
      const float xs[4] = {x.x, x.y, x.z, x.w};
      uint32_t t[3][4];
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const bf16_t b0 = from_f32<bf16_t>(xs[c]);
        const float r1 = xs[c] - static_cast<float>(b0);       // exact
        const bf16_t b1 = from_f32<bf16_t>(r1);
        const float r2 = r1 - static_cast<float>(b1);           // exact
        t[0][c] = (uint32_t)__builtin_bit_cast(uint16_t, b0);
        t[1][c] = (uint32_t)__builtin_bit_cast(uint16_t, b1);
        t[2][c] = bits(r2);
      }
#pragma unroll
      for (int m = 0; m < 3; ++m)
        *reinterpret_cast<uint2*>(&a_s[m][row][4 * q]) = make_uint2(t[m][0] | t[m][1] << 16, t[m][2] | t[m][3] << 16);
    }
#pragma unroll
    for (int i = 0; i < PSB; ++i) {
      const int e = tid + 256 * i, jn = e / (KCS / 8);
      if (e < GT * TN * (KCS / 8))
        *reinterpret_cast<u32x4*>(&b_s[jn / TN][jn % TN][8 * (e % (KCS / 8))]) = masked_piece(rb[i], keep_b >> i & 1u);
    }
    __syncthreads();
    int tap0, ntap, k0, base_off;
    stage_taps(stage, tap0, ntap, k0, base_off);
    if (stage + 1 < stages) fetch(stage + 1);
    for (int j = 0; j < ntap; ++j) {
      const int off = -(tap0 + j - half) * dil;
      const int shift = off - base_off;
      bool valid[U];
#pragma unroll
      for (int u = 0; u < U; ++u) valid[u] = tok[u] + off >= lo[u] && tok[u] + off < hi[u];
      // lane half hb supplies channels 8 hb .. 8 hb + 7 of its row (tokens) / column (outputs)
      u32x4 a[3][U];
#pragma unroll
      for (int m = 0; m < 3; ++m)
#pragma unroll
        for (int u = 0; u < U; ++u) a[m][u] = *reinterpret_cast<const u32x4*>(&a_s[m][row0 + 32 * u + ql + shift][8 * hb]);
      const u32x4 b = *reinterpret_cast<const u32x4*>(&b_s[j][col0 + ql][8 * hb]);
#pragma unroll
      for (int m = 2; m >= 0; --m)        // smallest terms first
#pragma unroll
        for (int u = 0; u < U; ++u) {
          a[m][u] = masked_piece(a[m][u], valid[u]);
          acc[u] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a[m][u]), __builtin_bit_cast(bf16x8, b),
                                                          acc[u], 0, 0, 0);
        }
    }
  }
  // accumulator register r of lane half hb: token row 8*(r/4) + 4*hb + r%4 of the sub-tile, output column ql
  const int n = n0 + col0 + ql;
  if (n >= N) return;
  auto token_of = [&](int ur) { return t0 + row0 + 32 * (ur / 16) + 8 * ((ur % 16) / 4) + 4 * hb + (ur % 4); };
  if (mode == 1) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      float pp[16];
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int64_t t = token_of(16 * u + r);
        pp[r] = pre_prev[t < total ? ((int64_t)h * total + t) * N + n : 0];
      }
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int64_t t = token_of(16 * u + r);
        if (t < total) out0[((int64_t)h * total + t) * N + n] = acc[u][r] * silu_grad_f32(pp[r]);
      }
    }
  } else {
    bf16_t* dst = n < D ? dk : dv;
    const int col = n < D ? n : n - D;
    if (dst != nullptr) {
#pragma unroll
      for (int ur = 0; ur < 16 * U; ++ur) {
        const int64_t t = token_of(ur);
        if (t < total) dst[(t * Hkv + h) * D + col] = from_f32<bf16_t>(acc[ur / 16][ur % 16]);
      }
    }
  }
}

// Stage 1 of d W_l: partial[chunk][h][c][m][tap] = sum over the chunk's tokens t of a_{l-1}[t + off][m] * d y_l[t][c],
// a tiled fp32 product with the tokens as the contraction index (slices of KCW tokens through LDS).  The chunk's
// sequence bounds are staged in LDS first, so a slice's operands need one round of global loads, not two dependent
// ones; the output channels are the rows of the matrix tiles, so neighbouring lanes write neighbouring m.
template <int WC, int WM>
__global__ void __launch_bounds__(256)
weight_product_kernel(const float* __restrict__ act_in, const float* __restrict__ dpre, int Cin, int Cout, int ks, int dil,
                      const int32_t* __restrict__ seq_lo, const int32_t* __restrict__ seq_hi, int64_t total, int Hkv,
                      int tiles_n, int tiles, int n_work, float* __restrict__ partial) {
  // [operand][token of the slice][channel ^ 32 * (token & 1)]: the two lane halves of an operand read take neighbouring
  // tokens, and the swap of the row halves on odd tokens puts them on different banks without padding the rows
  __shared__ float ab_s[2][KCW][64];
  float (*a_s)[64] = ab_s[0];          // activations, channel = m
  float (*b_s)[64] = ab_s[1];          // d y, channel = c
  __shared__ int32_t lo_s[kTokChunk], hi_s[kTokChunk];
  // Workgroups are dealt round-robin to the 8 XCDs; each XCD gets a contiguous range of work items, ordered (tile,
  // tap, head, chunk), so that the tiles and taps of one (head, chunk), which read the same rows, meet in one L2.
  const int per_xcd = (n_work + 7) / 8;
  const int work = ((int)blockIdx.x % 8) * per_xcd + (int)blockIdx.x / 8;
  if (work >= n_work) return;
  const int tile = work % tiles, head_tap = (work / tiles) % (Hkv * ks);
  const int m0 = (tile / tiles_n) * (32 * WM), c0 = (tile % tiles_n) * (32 * WC);
  const int h = head_tap / ks, tap = head_tap % ks;
  const int chunk = work / (tiles * Hkv * ks);
  const int tid = threadIdx.x;
  const int off = (tap - (ks - 1) / 2) * dil;
  const int64_t tb = (int64_t)chunk * kTokChunk;
  const int64_t te = tb + kTokChunk < total ? tb + kTokChunk : total;
  const float* a_h = act_in + (int64_t)h * total * Cin;
  const float* g_h = dpre + (int64_t)h * total * Cout;
  const int lane = tid & 63, wv = tid >> 6, ql = lane & 31, hb = lane >> 5;
  // Wave roles: WC x WM waves tile the output (32 output channels x 32 input channels each); when that takes fewer than
  // four, the S waves of a tile take every S-th pair of tokens of a slice and their sums are added in wave order.
  constexpr int S = 4 / (WC * WM);
  const int wq = wv % (WC * WM), sp = wv / (WC * WM), ci = wq / WM, mi = wq % WM;
  for (int i = tid; i < kTokChunk; i += 256) {
    const bool ok = tb + i < te;
    lo_s[i] = ok ? seq_lo[tb + i] : 0;
    hi_s[i] = ok ? seq_hi[tb + i] : 0;   // an empty range: rows past the chunk's end contribute nothing
  }
  __syncthreads();
  f32x16 acc;
#pragma unroll
  for (int r = 0; r < 16; ++r) acc[r] = 0.f;
  // A thread moves channel x of tokens wv, wv + 4, ... of a slice.  Token indices are kept relative to the chunk, in
  // 32 bits (the token count fits: the bounds are int32), so that a load costs little address arithmetic.
  const int x = tid & 63;
  const bool m_ok = x < 32 * WM && m0 + x < Cin, c_ok = x < 32 * WC && c0 + x < Cout;
  const float* a_col = a_h + tb * Cin + min(m0 + x, Cin - 1);
  const float* g_col = g_h + tb * Cout + min(c0 + x, Cout - 1);
  const int len = (int)(te - tb), tb32 = (int)tb;
  float ra[PERW], rb[PERW];
  unsigned keep_a, keep_b;     // one bit per loaded value: does it count
  auto fetch = [&](int i0) {
    keep_a = keep_b = 0u;
#pragma unroll
    for (int j = 0; j < PERW; ++j) {
      const int i = i0 + wv + 4 * j;                 // token of the chunk
      const bool t_ok = i < len;
      const int ic = t_ok ? i : 0;
      const int p = tb32 + ic + off;
      const bool p_ok = t_ok & (p >= lo_s[ic]) & (p < hi_s[ic]);
      // unconditional loads from rows inside the arrays; what does not count is zeroed where the value is consumed
      ra[j] = a_col[(int64_t)(p_ok ? ic + off : 0) * Cin];
      rb[j] = g_col[(int64_t)ic * Cout];
      keep_a |= (p_ok && m_ok) ? 1u << j : 0u;
      keep_b |= (t_ok && c_ok) ? 1u << j : 0u;
    }
  };
  fetch(0);
  for (int i0 = 0; i0 < len; i0 += KCW) {
    __syncthreads();
#pragma unroll
    for (int j = 0; j < PERW; ++j) {
      a_s[wv + 4 * j][x ^ ((wv & 1) << 5)] = masked_value(ra[j], keep_a >> j & 1u);      // token parity = wv & 1
      b_s[wv + 4 * j][x ^ ((wv & 1) << 5)] = masked_value(rb[j], keep_b >> j & 1u);
    }
    __syncthreads();
    if (i0 + KCW < len) fetch(i0 + KCW);   // the next slice's operands travel while this one is multiplied
#pragma unroll
    for (int tt = 2 * sp; tt < KCW; tt += 2 * S)
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(b_s[tt + hb][(32 * ci + ql) ^ (hb << 5)],
                                                 a_s[tt + hb][(32 * mi + ql) ^ (hb << 5)], acc, 0, 0, 0);   // tt is even
  }
  if constexpr (S > 1) {
    float* red = &ab_s[0][0][0];       // (S - 1) * WC * WM accumulator tiles of 1024 floats fit the operand tiles
    __syncthreads();
    if (sp > 0) {
#pragma unroll
      for (int r = 0; r < 16; ++r) red[((sp - 1) * WC * WM + wq) * 1024 + r * 64 + lane] = acc[r];
    }
    __syncthreads();
    if (sp > 0) return;
    for (int k = 1; k < S; ++k)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[r] += red[((k - 1) * WC * WM + wq) * 1024 + r * 64 + lane];
  }
  const int64_t per_head = (int64_t)Cout * Cin * ks;
  float* out = partial + ((int64_t)chunk * Hkv + h) * per_head;
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    const int c = c0 + 32 * ci + 8 * (r / 4) + 4 * hb + (r % 4);
    const int m = m0 + 32 * mi + ql;
    if (m < Cin && c < Cout) out[((int64_t)c * Cin + m) * ks + tap] = acc[r];     // the layout of the weights: [c][m][tap]
  }
}

// Stage 1 of d W_0 on bf16 storage: the input features are bf16 values, so with d y split into three bf16 terms (as in
// conv_back_bf16_kernel) three bf16 matrix instructions give the fp32 product.  The contraction runs over the tokens,
// i.e. over the rows of the staged [token][channel] tiles: both operands are fetched with transposing LDS loads
// (eight consecutive tokens of one channel per lane).  Rows are 96 elements apart, which spreads the four rows a
// 16-lane group reads over different banks.  Work order, wave roles and output as in weight_product_kernel with
// WM = 2 (2 D >= 128 input channels); a 64-channel tile of input channels lies in the keys or in the values.
constexpr int KCT = 64, RST = 96;            // tokens per slice, LDS row stride in elements
template <int WC>
__global__ void __launch_bounds__(256)
weight_first_bf16_kernel(const bf16_t* __restrict__ k, const bf16_t* __restrict__ v, int64_t stride_tok, int64_t stride_head,
                         const float* __restrict__ dpre, int D, int Cout, int ks, int dil,
                         const int32_t* __restrict__ seq_lo, const int32_t* __restrict__ seq_hi, int64_t total, int Hkv,
                         int tiles_n, int tiles, int n_work, float* __restrict__ partial) {
  __shared__ __align__(16) bf16_t x_s[KCT][RST];          // features: [token of the slice][m]
  __shared__ __align__(16) bf16_t g_s[3][KCT][RST];       // d y, term of the split: [token of the slice][c]
  __shared__ int32_t lo_s[kTokChunk], hi_s[kTokChunk];
  constexpr int WM = 2, S = 4 / (WC * WM);
  const int Cin = 2 * D;
  const int per_xcd = (n_work + 7) / 8;
  const int work = ((int)blockIdx.x % 8) * per_xcd + (int)blockIdx.x / 8;
  if (work >= n_work) return;
  const int tile = work % tiles, head_tap = (work / tiles) % (Hkv * ks);
  const int m0 = (tile / tiles_n) * 64, c0 = (tile % tiles_n) * (32 * WC);
  const int h = head_tap / ks, tap = head_tap % ks;
  const int chunk = work / (tiles * Hkv * ks);
  const int tid = threadIdx.x;
  const int off = (tap - (ks - 1) / 2) * dil;
  const int64_t tb = (int64_t)chunk * kTokChunk;
  const int64_t te = tb + kTokChunk < total ? tb + kTokChunk : total;
  const int len = (int)(te - tb), tb32 = (int)tb;
  const bf16_t* x_h = (m0 < D ? k + m0 : v + (m0 - D)) + (int64_t)h * stride_head;
  const float* g_h = dpre + ((int64_t)h * total + tb) * Cout;
  const int lane = tid & 63, wv = tid >> 6, hb = lane >> 5;
  const int wq = wv % (WC * WM), sp = wv / (WC * WM), ci = wq / WM, mi = wq % WM;
  for (int i = tid; i < kTokChunk; i += 256) {
    const bool ok = i < len;
    lo_s[i] = ok ? seq_lo[tb + i] : 0;
    hi_s[i] = ok ? seq_hi[tb + i] : 0;
  }
  __syncthreads();
  f32x16 acc;
#pragma unroll
  for (int r = 0; r < 16; ++r) acc[r] = 0.f;
  // loader roles: features as 16-byte pieces (8 per token row), d y as quads of floats (16 per token row)
  constexpr int PX = KCT * 8 / 256, PG = KCT * 16 / 256;
  u32x4 rx[PX];
  float4 rg[PG];
  unsigned keep_x, keep_g;
  auto fetch = [&](int i0) {
    keep_x = keep_g = 0u;
#pragma unroll
    for (int j = 0; j < PX; ++j) {
      const int e = tid + 256 * j, i = i0 + e / 8, q = e % 8;
      const bool t_ok = i < len;
      const int ic = t_ok ? i : 0;
      const int p = tb32 + ic + off;
      const bool p_ok = t_ok & (p >= lo_s[ic]) & (p < hi_s[ic]);
      rx[j] = *reinterpret_cast<const u32x4*>(x_h + (int64_t)(p_ok ? p : tb32) * stride_tok + 8 * q);
      keep_x |= p_ok ? 1u << j : 0u;
    }
#pragma unroll
    for (int j = 0; j < PG; ++j) {
      const int e = tid + 256 * j, i = i0 + e / 16, q = e % 16;
      const bool ok = i < len && c0 + 4 * q < Cout && 4 * q < 32 * WC;                // Cout % 4 == 0: whole quads
      rg[j] = *reinterpret_cast<const float4*>(g_h + (int64_t)(i < len ? i : 0) * Cout + min(c0 + 4 * q, Cout - 4));
      keep_g |= ok ? 1u << j : 0u;
    }
  };
  auto masked_piece = [](u32x4 x, bool keep) {
    asm volatile("" : "+v"(x));      // the loaded value is needed whatever the mask says: the load stays unconditional
    return keep ? x : u32x4{0u, 0u, 0u, 0u};
  };
  // transposing loads: in each group of 16 lanes, lane j points at row j / 4, columns 4 * (j % 4) .. of its 16 columns
  const int tr_row = 8 * hb + ((lane & 15) >> 2), tr_col = 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
  fetch(0);
  for (int i0 = 0; i0 < len; i0 += KCT) {
    __syncthreads();
#pragma unroll
    for (int j = 0; j < PX; ++j) {
      const int e = tid + 256 * j;
      *reinterpret_cast<u32x4*>(&x_s[e / 8][8 * (e % 8)]) = masked_piece(rx[j], keep_x >> j & 1u);
    }
#pragma unroll
    for (int j = 0; j < PG; ++j) {
      const int e = tid + 256 * j, row = e / 16, q = e % 16;
      const float4 y = masked_quad(rg[j], (keep_g >> j & 1u) ? 0xFu : 0u);
      const float ys[4] = {y.x, y.y, y.z, y.w};
      uint32_t t[3][4];
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const bf16_t b0 = from_f32<bf16_t>(ys[c]);
        const float r1 = ys[c] - static_cast<float>(b0);        // exact
        const bf16_t b1 = from_f32<bf16_t>(r1);
        const float r2 = r1 - static_cast<float>(b1);            // exact
        t[0][c] = (uint32_t)__builtin_bit_cast(uint16_t, b0);
        t[1][c] = (uint32_t)__builtin_bit_cast(uint16_t, b1);
        t[2][c] = (uint32_t)__builtin_bit_cast(uint16_t, from_f32<bf16_t>(r2));
      }
#pragma unroll
      for (int m = 0; m < 3; ++m)
        *reinterpret_cast<uint2*>(&g_s[m][row][4 * q]) = make_uint2(t[m][0] | t[m][1] << 16, t[m][2] | t[m][3] << 16);
    }
    __syncthreads();
    if (i0 + KCT < len) fetch(i0 + KCT);
#pragma unroll
    for (int st = sp; st < KCT / 16; st += S) {              // steps of 16 tokens, shared among the S waves of a tile
      const bf16x8 b = load_transposed(&x_s[16 * st + tr_row][32 * mi + tr_col], RST);
#pragma unroll
      for (int m = 2; m >= 0; --m)                           // smallest terms first
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(load_transposed(&g_s[m][16 * st + tr_row][32 * ci + tr_col], RST), b,
                                                      acc, 0, 0, 0);
    }
  }
  if constexpr (S > 1) {
    float* red = reinterpret_cast<float*>(&g_s[0][0][0]);   // (S - 1) * WC * WM accumulator tiles of 1024 floats
    __syncthreads();
    if (sp > 0) {
#pragma unroll
      for (int r = 0; r < 16; ++r) red[((sp - 1) * WC * WM + wq) * 1024 + r * 64 + lane] = acc[r];
    }
    __syncthreads();
    if (sp > 0) return;
    for (int kk = 1; kk < S; ++kk)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[r] += red[((kk - 1) * WC * WM + wq) * 1024 + r * 64 + lane];
  }
  const int64_t per_head = (int64_t)Cout * Cin * ks;
  float* out = partial + ((int64_t)chunk * Hkv + h) * per_head;
  const int ql = lane & 31;
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    const int c = c0 + 32 * ci + 8 * (r / 4) + 4 * hb + (r % 4);
    const int m = m0 + 32 * mi + ql;
    if (m < Cin && c < Cout) out[((int64_t)c * Cin + m) * ks + tap] = acc[r];
  }
}

// Stage 2: out[i] = sum over chunks of partial[chunk][i], in chunk order.
__global__ void __launch_bounds__(256)
chunk_sum_kernel(const float* __restrict__ partial, int64_t n, int chunks, float* __restrict__ out) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n) return;
  float acc = 0.f;
#pragma unroll 8
  for (int ch = 0; ch < chunks; ++ch) acc += partial[(int64_t)ch * n + i];
  out[i] = acc;
}

// Stage 2 of every sum of a call in one launch: blockIdx.y picks the sum, out[i] = sum over its chunks in chunk order.
constexpr int kMaxSums = 2 * LTEA_MAX_CNN_LAYERS + 2;
struct SumSeg { const float* partial; float* out; int64_t n; int chunks; };
struct SumSegs { SumSeg s[kMaxSums]; };
__global__ void __launch_bounds__(256)
chunk_sum_all_kernel(const SumSegs S) {
  const SumSeg seg = S.s[blockIdx.y];
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= seg.n) return;
  float acc = 0.f;
#pragma unroll 8
  for (int ch = 0; ch < seg.chunks; ++ch) acc += seg.partial[(int64_t)ch * seg.n + i];
  seg.out[i] = acc;
}

// Column sums over the tokens: out[h][c] = sum_t x[h][t][c] (mode 0), sum_t dz[h][t] * x[h][t][c] (mode 1),
// or, with C = 1, sum_t dz[h][t] (mode 2).  One workgroup per (h, tile of c_tile channels, c_tile a power of two
// <= 64) and chunk of kColChunk tokens: 256 / c_tile token lanes each sum a strided share in order (neighbouring
// threads read neighbouring channels of one token), then the lanes of a channel are added in lane order; the chunks
// are added by chunk_sum_kernel.
__global__ void __launch_bounds__(256)
column_sum_kernel(const float* __restrict__ x, const float* __restrict__ dz, int C, int c_tile, int64_t total, int mode,
                  int Hkv, float* __restrict__ partial) {
  __shared__ float red[256];
  const int h = blockIdx.y;
  const int lanes = 256 / c_tile;
  const int c = blockIdx.x * c_tile + (int)threadIdx.x % c_tile, tl = (int)threadIdx.x / c_tile;
  float acc = 0.f;
  if (c < C) {
    const int64_t tb = (int64_t)blockIdx.z * kColChunk;
    const int64_t te = tb + kColChunk < total ? tb + kColChunk : total;
#pragma unroll 8
    for (int64_t t = tb + tl; t < te; t += lanes) {
      const float g = dz != nullptr ? dz[(int64_t)h * total + t] : 1.0f;
      if (mode == 2) acc += g;
      else {
        const float xv = x[((int64_t)h * total + t) * C + c];
        acc += mode == 1 ? g * xv : xv;
      }
    }
  }
  red[threadIdx.x] = acc;
  __syncthreads();
  if (tl == 0 && c < C) {
    float sum = 0.f;
    for (int j = 0; j < lanes; ++j) sum += red[j * c_tile + (int)threadIdx.x];
    partial[((int64_t)blockIdx.z * Hkv + h) * C + c] = sum;
  }
}

size_t up256(size_t x) { return (x + 255) / 256 * 256; }

struct Layout {
  int32_t *seq_lo, *seq_hi;
  float* a0;                                  // [Hkv][T][2D] input features as fp32
  float* pre[LTEA_MAX_CNN_LAYERS];            // [Hkv][T][C_l]
  float* act[LTEA_MAX_CNN_LAYERS];
  float* dpre[2];                             // [Hkv][T][widest layer], ping-pong
  float *wf[LTEA_MAX_CNN_LAYERS], *wb[LTEA_MAX_CNN_LAYERS];   // fp32 weight panels of every layer
  void* wq0;                                  // first layer's weights [Hkv][k][C_0][2D] in the storage type (bf16 only)
  void* wqf[LTEA_MAX_CNN_LAYERS];             // every layer's weights [Hkv][k][C_{l-1}][C_l] in the storage type (bf16 only)
  float* part_w[LTEA_MAX_CNN_LAYERS];         // [chunks][Hkv][C_l][C_{l-1}][k]: partial weight gradients
  float* part_b[LTEA_MAX_CNN_LAYERS];         // [column chunks][Hkv][C_l]: partial bias gradients
  float *part_wout, *part_bout;               // [column chunks][Hkv][C_L], [column chunks][Hkv]
  size_t bytes;
};

Layout carve(const ltea_cfg& cfg, const ltea_cnn& cnn, int64_t total, void* base) {
  Layout L;
  uintptr_t p = reinterpret_cast<uintptr_t>(base);   // integer arithmetic: a size query carves from a null base
  auto take = [&](size_t bytes) { char* r = reinterpret_cast<char*>(p); p += up256(bytes); return r; };
  const size_t rows = (size_t)cfg.Hkv * (size_t)total;
  L.seq_lo = reinterpret_cast<int32_t*>(take(sizeof(int32_t) * (size_t)total));
  L.seq_hi = reinterpret_cast<int32_t*>(take(sizeof(int32_t) * (size_t)total));
  L.a0 = reinterpret_cast<float*>(take(sizeof(float) * rows * 2 * cfg.D));
  int cmax = 0;
  int cin = 2 * cfg.D;
  for (int l = 0; l < LTEA_MAX_CNN_LAYERS; ++l) L.pre[l] = L.act[l] = nullptr;
  for (int l = 0; l < cnn.n_layers; ++l) {
    L.pre[l] = reinterpret_cast<float*>(take(sizeof(float) * rows * cnn.c_out[l]));
    L.act[l] = reinterpret_cast<float*>(take(sizeof(float) * rows * cnn.c_out[l]));
    cmax = cnn.c_out[l] > cmax ? cnn.c_out[l] : cmax;
    cin = cnn.c_out[l];
  }
  for (int i = 0; i < 2; ++i) L.dpre[i] = reinterpret_cast<float*>(take(sizeof(float) * rows * cmax));
  cin = 2 * cfg.D;
  for (int l = 0; l < LTEA_MAX_CNN_LAYERS; ++l) L.wf[l] = L.wb[l] = nullptr;
  for (int l = 0; l < cnn.n_layers; ++l) {
    const size_t w = (size_t)cfg.Hkv * cnn.c_out[l] * cin * cnn.kernel[l];
    L.wf[l] = reinterpret_cast<float*>(take(sizeof(float) * w));
    L.wb[l] = reinterpret_cast<float*>(take(sizeof(float) * w));
    cin = cnn.c_out[l];
  }
  cin = 2 * cfg.D;
  for (int l = 0; l < LTEA_MAX_CNN_LAYERS; ++l) L.wqf[l] = nullptr;
  for (int l = 0; l < cnn.n_layers; ++l) {
    if (cfg.dtype != LTEA_F32) L.wqf[l] = take(sizeof(bf16_t) * (size_t)cfg.Hkv * cnn.c_out[l] * cin * cnn.kernel[l]);
    cin = cnn.c_out[l];
  }
  L.wq0 = cfg.dtype == LTEA_F32 ? nullptr : take(sizeof(bf16_t) * (size_t)cfg.Hkv * cnn.c_out[0] * 2 * cfg.D * cnn.kernel[0]);
  const size_t chunks = (size_t)((total + kTokChunk - 1) / kTokChunk);
  const size_t col_chunks = (size_t)((total + kColChunk - 1) / kColChunk);
  cin = 2 * cfg.D;
  for (int l = 0; l < LTEA_MAX_CNN_LAYERS; ++l) L.part_w[l] = L.part_b[l] = nullptr;
  for (int l = 0; l < cnn.n_layers; ++l) {
    L.part_w[l] = reinterpret_cast<float*>(take(sizeof(float) * chunks * cfg.Hkv * cnn.c_out[l] * cin * cnn.kernel[l]));
    L.part_b[l] = reinterpret_cast<float*>(take(sizeof(float) * col_chunks * cfg.Hkv * cnn.c_out[l]));
    cin = cnn.c_out[l];
  }
  L.part_wout = reinterpret_cast<float*>(take(sizeof(float) * col_chunks * cfg.Hkv * cin));
  L.part_bout = reinterpret_cast<float*>(take(sizeof(float) * col_chunks * cfg.Hkv));
  L.bytes = (size_t)(p - reinterpret_cast<uintptr_t>(base));
  return L;
}

template <typename T>
hipError_t run(const ltea_cfg& cfg, const ltea_cnn& cnn, const void* k, const void* v, int64_t stride_tok,
               int64_t stride_head, const SeqView& sv, const float* dz, const ltea_cnn_grad& g, void* dk, void* dv,
               void* workspace, hipStream_t stream) {
  const int64_t total = sv.total_tokens;
  const int Hkv = cfg.Hkv, nl = cnn.n_layers, D = cfg.D;
  const Layout L = carve(cfg, cnn, total, workspace);
  hipError_t e;
  const unsigned tok_tiles = (unsigned)((total + TMC - 1) / TMC);
  auto blocks = [](int64_t n) { return dim3((unsigned)((n + 255) / 256)); };
  auto cin_of = [&](int l) { return l == 0 ? 2 * D : cnn.c_out[l - 1]; };
  auto in_of = [&](int l) -> const float* { return l == 0 ? L.a0 : L.act[l - 1]; };
  // rows of both operands in whole, 16-byte aligned quads: the vector-load instance
  auto conv_product = [](int K, int N) {
    const bool vec = K % 4 == 0 && N % 4 == 0;
    if (N <= 32) return vec ? conv_product_kernel<T, true, true> : conv_product_kernel<T, false, true>;
    return vec ? conv_product_kernel<T, true, false> : conv_product_kernel<T, false, false>;
  };
  auto panels = [&](int l) {
    const int64_t n = (int64_t)Hkv * cnn.c_out[l] * cin_of(l) * cnn.kernel[l];
    hipLaunchKernelGGL(weight_panels_kernel<T>, blocks(n), dim3(256), 0, stream, static_cast<const T*>(cnn.w[l]), cin_of(l),
                       cnn.c_out[l], cnn.kernel[l], n, L.wf[l], L.wb[l],
                       l == 0 ? static_cast<T*>(L.wq0) : static_cast<T*>(nullptr), static_cast<T*>(L.wqf[l]));
    return hipGetLastError();
  };
  hipLaunchKernelGGL(token_bounds_kernel, blocks(total), dim3(256), 0, stream, sv.cu_seqlens, sv.n_seqs, total, L.seq_lo,
                     L.seq_hi);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  // on bf16 storage the first layer's kernels read k / v themselves, unless its weight product takes the fp32 route
  if (!(std::is_same<T, bf16_t>::value && cnn.c_out[0] % 4 == 0)) {
    hipLaunchKernelGGL(features_kernel<T>, dim3((unsigned)((total * (2 * D / Elems<T>::N) + 255) / 256), (unsigned)Hkv), dim3(256),
                       0, stream, static_cast<const T*>(k), static_cast<const T*>(v), stride_tok, stride_head, D, total, L.a0);
  }
  if ((e = hipGetLastError()) != hipSuccess) return e;
  // 1. forward, pre-activations and activations kept
  for (int l = 0; l < nl; ++l) {
    if ((e = panels(l)) != hipSuccess) return e;
    const int N = cnn.c_out[l];
    if constexpr (std::is_same<T, bf16_t>::value) {
      if (l == 0) {     // both operands are bf16 values: the bf16 matrix instruction gives the fp32 result
        const dim3 grid(tok_tiles, (unsigned)((N + TN - 1) / TN), (unsigned)Hkv);
        hipLaunchKernelGGL(N <= 32 ? conv_first_bf16_kernel<true> : conv_first_bf16_kernel<false>, grid, dim3(256), 0, stream,
                           static_cast<const bf16_t*>(k), static_cast<const bf16_t*>(v), stride_tok, stride_head,
                           static_cast<const bf16_t*>(L.wq0), D, N, cnn.kernel[0], cnn.dilation[0], L.seq_lo, L.seq_hi, total,
                           cnn.bias[0], L.pre[0], L.act[0]);
        if ((e = hipGetLastError()) != hipSuccess) return e;
        continue;
      }
    }
    hipLaunchKernelGGL(conv_product(cin_of(l), N), dim3(tok_tiles, (unsigned)((N + TN - 1) / TN), (unsigned)Hkv), dim3(256), 0,
                       stream, in_of(l), L.wf[l], cin_of(l), N, cnn.kernel[l], cnn.dilation[l], 1, L.seq_lo, L.seq_hi, total,
                       Hkv, 0, cnn.bias[l], static_cast<const float*>(nullptr), L.pre[l], L.act[l], static_cast<T*>(nullptr),
                       static_cast<T*>(nullptr), D);
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  // 2. output projection
  const int CL = cnn.c_out[nl - 1];
  hipLaunchKernelGGL(out_proj_backward_kernel<T>, dim3((unsigned)((total * CL + 255) / 256), (unsigned)Hkv), dim3(256), 0,
                     stream, dz, static_cast<const T*>(cnn.w_out), L.pre[nl - 1], CL, total, L.dpre[0]);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  auto c_tile_of = [](int C) { int t = 1; while (t < C && t < 64) t *= 2; return t; };
  const int chunks = (int)((total + kTokChunk - 1) / kTokChunk);
  const int col_chunks = (int)((total + kColChunk - 1) / kColChunk);
  // every sum's second stage runs in one launch at the end
  SumSegs sums;
  int n_sums = 0;
  int64_t n_sum_max = 0;
  auto second_stage = [&](const float* partial, float* out, int64_t n, int n_chunks) {
    sums.s[n_sums++] = SumSeg{partial, out, n, n_chunks};
    n_sum_max = n > n_sum_max ? n : n_sum_max;
  };
  auto column_sum = [&](const float* x, const float* dzp, int C, int mode, float* partial, float* out) {
    const int ct = c_tile_of(C);
    hipLaunchKernelGGL(column_sum_kernel, dim3((unsigned)((C + ct - 1) / ct), (unsigned)Hkv, (unsigned)col_chunks), dim3(256),
                       0, stream, x, dzp, C, ct, total, mode, Hkv, partial);
    second_stage(partial, out, (int64_t)Hkv * C, col_chunks);
    return hipGetLastError();
  };
  if ((e = column_sum(L.act[nl - 1], dz, CL, 1, L.part_wout, g.w_out)) != hipSuccess) return e;
  if ((e = column_sum(nullptr, dz, 1, 2, L.part_bout, g.b_out)) != hipSuccess) return e;
  // 3. layers in reverse
  int cur = 0;
  for (int l = nl - 1; l >= 0; --l) {
    const int Cout = cnn.c_out[l], Cin = cin_of(l), ks = cnn.kernel[l];
    const float* dpre = L.dpre[cur];
    if ((e = column_sum(dpre, nullptr, Cout, 0, L.part_b[l], g.bias[l])) != hipSuccess) return e;
    // 32-wide halves of the 64 x 64 tile that a narrow layer would leave empty go to sharing the tokens instead
    const int wc = Cout <= 32 ? 1 : 2, wm = Cin <= 32 ? 1 : 2;
    const int tiles_m = (Cin + 32 * wm - 1) / (32 * wm), tiles_n = (Cout + 32 * wc - 1) / (32 * wc);
    auto weight_product = wc == 2 ? (wm == 2 ? weight_product_kernel<2, 2> : weight_product_kernel<2, 1>)
                                  : (wm == 2 ? weight_product_kernel<1, 2> : weight_product_kernel<1, 1>);
    const int64_t n_work = (int64_t)tiles_m * tiles_n * Hkv * ks * chunks;
    if (n_work > (int64_t)1 << 30) return hipErrorInvalidValue;
    if constexpr (std::is_same<T, bf16_t>::value) {
      if (l == 0 && Cout % 4 == 0) {   // bf16 features, d y split into three bf16 terms
        hipLaunchKernelGGL(wc == 2 ? weight_first_bf16_kernel<2> : weight_first_bf16_kernel<1>, dim3((unsigned)((n_work + 7) / 8 * 8)),
                           dim3(256), 0, stream, static_cast<const bf16_t*>(k), static_cast<const bf16_t*>(v), stride_tok,
                           stride_head, dpre, D, Cout, ks, cnn.dilation[0], L.seq_lo, L.seq_hi, total, Hkv, tiles_n,
                           tiles_m * tiles_n, (int)n_work, L.part_w[0]);
        if ((e = hipGetLastError()) != hipSuccess) return e;
        second_stage(L.part_w[0], g.w[0], (int64_t)Cout * Cin * ks * Hkv, chunks);
        goto weights_done;
      }
    }
    hipLaunchKernelGGL(weight_product, dim3((unsigned)((n_work + 7) / 8 * 8)), dim3(256), 0, stream, in_of(l), dpre, Cin, Cout,
                       ks, cnn.dilation[l], L.seq_lo, L.seq_hi, total, Hkv, tiles_n, tiles_m * tiles_n, (int)n_work, L.part_w[l]);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    second_stage(L.part_w[l], g.w[l], (int64_t)Cout * Cin * ks * Hkv, chunks);
  weights_done:
    if (l > 0 || dk != nullptr || dv != nullptr) {
      // towards the input: contraction over this layer's output channels, taps mirrored
      bool done = false;
      if constexpr (std::is_same<T, bf16_t>::value) {
        if (Cout % 8 == 0 && Cin % 8 == 0) {   // bf16 weights, d y split into three bf16 terms
          const dim3 grid(tok_tiles, (unsigned)((Cin + TN - 1) / TN), (unsigned)Hkv);
          hipLaunchKernelGGL(Cin <= 32 ? conv_back_bf16_kernel<true> : conv_back_bf16_kernel<false>, grid, dim3(256), 0, stream,
                             dpre, static_cast<const bf16_t*>(L.wqf[l]), Cout, Cin, ks, cnn.dilation[l], L.seq_lo, L.seq_hi,
                             total, Hkv, l > 0 ? 1 : 2, l > 0 ? L.pre[l - 1] : static_cast<const float*>(nullptr),
                             L.dpre[cur ^ 1], static_cast<bf16_t*>(dk), static_cast<bf16_t*>(dv), D);
          if ((e = hipGetLastError()) != hipSuccess) return e;
          done = true;
        }
      }
      if (!done) {
      hipLaunchKernelGGL(conv_product(Cout, Cin), dim3(tok_tiles, (unsigned)((Cin + TN - 1) / TN), (unsigned)Hkv), dim3(256), 0,
                         stream, dpre, L.wb[l], Cout, Cin, ks, cnn.dilation[l], -1, L.seq_lo, L.seq_hi, total, Hkv,
                         l > 0 ? 1 : 2, static_cast<const float*>(nullptr),
                         l > 0 ? L.pre[l - 1] : static_cast<const float*>(nullptr), L.dpre[cur ^ 1],
                         static_cast<float*>(nullptr), static_cast<T*>(dk), static_cast<T*>(dv), D);
      if ((e = hipGetLastError()) != hipSuccess) return e;
      }
    }
    cur ^= 1;
  }
  hipLaunchKernelGGL(chunk_sum_all_kernel, dim3((unsigned)((n_sum_max + 255) / 256), (unsigned)n_sums), dim3(256), 0, stream, sums);
  return hipGetLastError();
}

}  // namespace

size_t cnn_backward_workspace(const ltea_cfg& cfg, const ltea_cnn& cnn, int64_t total_tokens) {
  return carve(cfg, cnn, total_tokens, nullptr).bytes;
}

hipError_t launch_cnn_backward(const ltea_cfg& cfg, const ltea_cnn& cnn, const void* k, const void* v,
                               int64_t stride_tok, int64_t stride_head, const SeqView& sv, const float* dz,
                               const ltea_cnn_grad& grad, void* dk, void* dv, void* workspace, hipStream_t stream) {
  if (sv.total_tokens == 0) {   // no tokens: every gradient is zero (a sum over no chunks)
    auto zero = [&](float* out, int64_t n) {
      hipLaunchKernelGGL(chunk_sum_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream,
                         static_cast<const float*>(nullptr), n, 0, out);
    };
    int cin = 2 * cfg.D;
    for (int l = 0; l < cnn.n_layers; ++l) {
      zero(grad.w[l], (int64_t)cfg.Hkv * cnn.c_out[l] * cin * cnn.kernel[l]);
      zero(grad.bias[l], (int64_t)cfg.Hkv * cnn.c_out[l]);
      cin = cnn.c_out[l];
    }
    zero(grad.w_out, (int64_t)cfg.Hkv * cin);
    zero(grad.b_out, cfg.Hkv);
    return hipGetLastError();
  }
  if (cfg.dtype == LTEA_F32)
    return run<float>(cfg, cnn, k, v, stride_tok, stride_head, sv, dz, grad, dk, dv, workspace, stream);
  return run<bf16_t>(cfg, cnn, k, v, stride_tok, stride_head, sv, dz, grad, dk, dv, workspace, stream);
}

}  // namespace ltea
