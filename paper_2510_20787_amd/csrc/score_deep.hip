// Scoring CNN of the LTE module with several convolution layers (paper Section 3.1.1, Appendix A: three k = 3,
// dilation-2 layers halving the channels, receptive field 13), fused into one bf16 MFMA kernel.
//
//   a_0[j] = concat(key_j, value_j);  a_l[j][c] = Swish( bias_l[c] + sum_{t,m} W_l[c][m][t] * a_{l-1}[j + (t-half_l)*dil_l][m] )
//   z[j] = b_out + sum_c w_out[c] * a_L[j][c];   activations of positions outside the sequence are zero at every layer.
//
// One workgroup (4 waves) = one tile of one (sequence, KV head).  Every layer computes 128 consecutive positions
// (32 per wave, the MFMA column dimension; output channels are the MFMA rows), anchored so that the positions a
// later layer needs are inside what the earlier one produced: layer l covers positions j0 - h_l .. j0 - h_l + 127
// with h_l the half receptive field of the layers after l.  Of the last layer's 128 positions the first
// TM = 128 - 2*h_1 have exact inputs and are written.
//
// Layer 1 contracts over the 2*D input channels in chunks of 32: the chunk's token rows (with halo; rows outside
// the sequence read as zeros through a range-limited buffer descriptor) and the chunk's tap-major weight panels
// are prefetched into registers during the previous chunk's MFMAs and then stored to LDS.  Intermediate
// activations stay in LDS and never touch HBM.  They are fp32 values kept as two bf16 terms (hi + lo, 16
// mantissa bits together), each multiplied by the bf16 weights in its own MFMA, so that the logits keep fp32-level
// accuracy: retention compares logits, and rounding activations to one bf16 would move them by ~1e-3.
// Activation buffers of consecutive layers alternate between two LDS regions; the second one reuses the space of
// layer 1's chunk buffers.  Weight panels of layers >= 2 are staged into a third region when their layer starts.
#include "ltea_common.h"
#include "ltea_kernels.h"

namespace ltea {
namespace {

constexpr int kThreads = 256;
constexpr int kPos = 128;     // positions per layer per workgroup
constexpr int CK = 32;        // input channels per chunk of layer 1
constexpr int XS1 = CK + 8;   // LDS row stride (elements) of layer 1's chunk buffers
constexpr int kMaxL = LTEA_MAX_CNN_LAYERS;
constexpr int kMaxXPieces = 3;   // 16-byte pieces of the token chunk per thread  (rows <= 192)
constexpr int kMaxWPieces = 7;   // 16-byte pieces of the weight chunk per thread (taps * padded channels <= 448)

struct DeepArgs {
  const bf16_t* k; const bf16_t* v; int64_t st, sh;
  const bf16_t* panels;          // [layer][Hkv][tap][cp][cin], channels zero-padded to cp
  int64_t panel_off[kMaxL];      // element offset of layer l's block
  int64_t panel_head[kMaxL];     // elements per head in layer l's block
  const float* bias[kMaxL];
  const bf16_t* w_out; const float* b_out;
  int L, ks[kMaxL], dil[kMaxL], cin[kMaxL], cout[kMaxL], cp[kMaxL];
  int TM, x_rows;                // valid tokens per tile; token rows of layer 1's chunk buffer
  int h0;                        // half receptive field of the whole stack
  int lds_ra, lds_r1, lds_rw;    // element offsets of the three LDS regions
  const int32_t* cu; int n_seqs; int64_t total; float* logits;
};

struct PanelArgs {
  const uint16_t* w[kMaxL]; int64_t off[kMaxL], total[kMaxL]; int cout[kMaxL], cp[kMaxL], cin[kMaxL], ks[kMaxL];
};

// panels[l][h][tap][c][m] = W_l[h][c][m][tap] for c < cout, 0 for cout <= c < cp; blockIdx.y = layer
__global__ void __launch_bounds__(256)
deep_panels_kernel(PanelArgs a, uint16_t* __restrict__ panels) {
  const int l = blockIdx.y;
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;   // over [Hkv][ks][cp][cin] of layer l
  if (idx >= a.total[l]) return;
  const int cin = a.cin[l], cp = a.cp[l], ks = a.ks[l], cout = a.cout[l];
  const int m = (int)(idx % cin);
  int64_t r = idx / cin;
  const int c = (int)(r % cp); r /= cp;
  const int tap = (int)(r % ks);
  const int64_t h = r / ks;
  panels[a.off[l] + idx] = c < cout ? a.w[l][((h * cout + c) * cin + m) * ks + tap] : (uint16_t)0;
}

__global__ void __launch_bounds__(kThreads, 2)
score_deep_kernel(const DeepArgs a) {
  extern __shared__ __align__(16) unsigned char smem[];
  bf16_t* lds = reinterpret_cast<bf16_t*>(smem);

  const int h = blockIdx.y;
  int tile, s, n, lo32;
  if (!locate_tile(a.cu, a.n_seqs, a.TM, blockIdx.x, s, tile, lo32, n)) return;
  const int64_t lo = lo32;
  const int j0 = tile * a.TM;
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, ql = lane & 31, hb = lane >> 5;
  const int row = 32 * wv + ql;             // this lane's position index inside every layer's 128

  // ================= layer 1: contraction over 2*D input channels in chunks of CK ==========================
  const int ks1 = a.ks[0], dil1 = a.dil[0], cp1 = a.cp[0], c2 = a.cin[0], D = c2 / 2;
  bf16_t* x_lds = lds + a.lds_r1;
  bf16_t* w_lds = x_lds + a.x_rows * XS1;
  // Descriptors start at the first row this tile reads (the sequence start when the halo reaches before it: those
  // rows wrap to huge offsets) and end at the last one or at the sequence end: 32-bit byte offsets span one tile.
  const uint32_t row_bytes = (uint32_t)a.st * 2u;
  const int base_row = j0 >= a.h0 ? j0 - a.h0 : 0;
  const int rows_here = n - base_row < a.x_rows ? n - base_row : a.x_rows;
  const uint32_t seq_bytes = (uint32_t)(rows_here - 1) * row_bytes + (uint32_t)(D * 2);
  const int64_t base_el = (lo + base_row) * a.st + (int64_t)h * a.sh;
  const auto rs_k = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t*>(a.k + base_el), 0, seq_bytes, 0x00020000);
  const auto rs_v = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t*>(a.v + base_el), 0, seq_bytes, 0x00020000);
  const uint32_t w1_bytes = (uint32_t)(ks1 * cp1 * c2) * 2u;
  const auto rs_w = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<bf16_t*>(a.panels + a.panel_off[0] + (int64_t)h * a.panel_head[0]), 0, w1_bytes, 0x00020000);
  const int n_xp = a.x_rows * (CK / 8), n_wp = ks1 * cp1 * (CK / 8);   // 16-byte pieces per chunk
  u32x4 xreg[kMaxXPieces], wreg[kMaxWPieces];
  auto load_chunk = [&](int chunk) {
    const int c0 = chunk * CK;
    const bool from_v = c0 >= D;
    const uint32_t col = (uint32_t)((from_v ? c0 - D : c0) * 2);
#pragma unroll
    for (int i = 0; i < kMaxXPieces; ++i) {
      const int p = tid + i * kThreads, r = p >> 2, pc = p & 3;
      // rows before the sequence wrap to huge offsets and rows past its end are beyond the range: both read zeros
      const uint32_t off = (uint32_t)(j0 - a.h0 + r - base_row) * row_bytes + col + (uint32_t)pc * 16u;
      xreg[i] = from_v ? __builtin_amdgcn_raw_buffer_load_b128(rs_v, off, 0, 0)
                       : __builtin_amdgcn_raw_buffer_load_b128(rs_k, off, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < kMaxWPieces; ++i) {
      const int p = tid + i * kThreads, r = p >> 2, pc = p & 3;           // r = tap*cp1 + c
      const uint32_t off = (uint32_t)(r * c2 + c0 + pc * 8) * 2u;         // past the panels -> zeros (never stored)
      wreg[i] = __builtin_amdgcn_raw_buffer_load_b128(rs_w, off, 0, 0);
    }
  };
  auto store_chunk = [&]() {
#pragma unroll
    for (int i = 0; i < kMaxXPieces; ++i) {
      const int p = tid + i * kThreads;
      if (p < n_xp) *reinterpret_cast<u32x4*>(&x_lds[(p >> 2) * XS1 + (p & 3) * 8]) = xreg[i];
    }
#pragma unroll
    for (int i = 0; i < kMaxWPieces; ++i) {
      const int p = tid + i * kThreads;
      if (p < n_wp) *reinterpret_cast<u32x4*>(&w_lds[(p >> 2) * XS1 + (p & 3) * 8]) = wreg[i];
    }
  };

  f32x16 acc[2];
#pragma unroll
  for (int mb = 0; mb < 2; ++mb)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[mb][r] = 0.f;

  const int n_chunks = c2 / CK;
  load_chunk(0);
  for (int chunk = 0; chunk < n_chunks; ++chunk) {
    if (chunk > 0) __syncthreads();        // the previous chunk's buffers are no longer read
    store_chunk();
    __syncthreads();
    if (chunk + 1 < n_chunks) load_chunk(chunk + 1);
    for (int tap = 0; tap < ks1; ++tap) {
      const bf16_t* b_row = x_lds + (row + tap * dil1) * XS1 + 8 * hb;
      const bf16_t* a_row = w_lds + (tap * cp1 + ql) * XS1 + 8 * hb;
#pragma unroll
      for (int kk = 0; kk < CK / 16; ++kk) {
        const bf16x8 b = *reinterpret_cast<const bf16x8*>(b_row + 16 * kk);
        const bf16x8 a0 = *reinterpret_cast<const bf16x8*>(a_row + 16 * kk);
        acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, b, acc[0], 0, 0, 0);
        if (cp1 > 32) {
          const bf16x8 a1 = *reinterpret_cast<const bf16x8*>(a_row + 32 * XS1 + 16 * kk);
          acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, b, acc[1], 0, 0, 0);
        }
      }
    }
  }

  // Swish(acc + bias) of layer l; accumulator register r of block mb is channel 32*mb + 8*(r/4) + 4*hb + r%4
  auto activation = [&](int l, int mb, int g4, float (&y)[4]) {
    const int c = 32 * mb + 8 * g4 + 4 * hb;
    const int cout = a.cout[l];
    const float* bl = a.bias[l] + (int64_t)h * cout;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int cc = c + e < cout ? c + e : cout - 1;      // unconditional load, then select
      const float x = acc[mb][4 * g4 + e] + bl[cc];
      const float sw = x * __frcp_rn(1.0f + __expf(-x));
      y[e] = c + e < cout ? sw : 0.f;
    }
  };

  // Stores layer l's activations (zero outside the sequence) as hi + lo bf16 rows of stride cout + 8.
  auto store_activations = [&](int l, bf16_t* dst, int h_l) {
    const int cout = a.cout[l], as = cout + 8;
    const int pos = j0 - h_l + row;
    const bool inside = pos >= 0 && pos < n;
    bf16_t* hi_row = dst + row * as;
    bf16_t* lo_row = dst + (kPos + row) * as;
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {
        const int c = 32 * mb + 8 * g4 + 4 * hb;
        if (c < cout) {                      // cout is a multiple of 16, so a group of 4 is all in or all out
          float y[4];
          activation(l, mb, g4, y);
          bf16x4 hi, lw;
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const float val = inside ? y[e] : 0.f;
            hi[e] = static_cast<bf16_t>(val);
            lw[e] = static_cast<bf16_t>(val - static_cast<float>(hi[e]));
          }
          *reinterpret_cast<bf16x4*>(hi_row + c) = hi;
          *reinterpret_cast<bf16x4*>(lo_row + c) = lw;
        }
      }
  };

  // ================= layers 2 .. L ============================================================================
  int h_prev = a.h0 - (ks1 - 1) / 2 * dil1;    // h_1
  bf16_t* act_a = lds + a.lds_ra;
  bf16_t* act_b = lds + a.lds_r1;
  bf16_t* w2_lds = lds + a.lds_rw;
  __syncthreads();                             // layer 1's chunk buffers are free (act_b aliases them)
  bf16_t* act_in = act_a;
  if (a.L > 1) store_activations(0, act_in, h_prev);
  for (int l = 1; l < a.L; ++l) {
    const int ksl = a.ks[l], dl = a.dil[l], cpl = a.cp[l], cinl = a.cin[l], ws = cinl + 8, as = cinl + 8;
    // stage this layer's panels (all taps): rows of cinl elements -> padded rows
    if (l > 1) __syncthreads();                // the previous layer's panels are no longer read
    {
      const int ppr = cinl / 8, n_p = ksl * cpl * ppr;
      const u32x4* src = reinterpret_cast<const u32x4*>(a.panels + a.panel_off[l] + (int64_t)h * a.panel_head[l]);
      for (int p = tid; p < n_p; p += kThreads) {
        const int r = p / ppr, pc = p - r * ppr;
        *reinterpret_cast<u32x4*>(&w2_lds[r * ws + pc * 8]) = src[p];
      }
    }
    __syncthreads();                           // panels and the previous layer's activations are visible
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[mb][r] = 0.f;
    for (int tap = 0; tap < ksl; ++tap) {
      int rr = row + tap * dl;                 // input row of this position; rows past 127 belong to positions
      rr = rr < kPos ? rr : kPos - 1;          //   whose results are dropped: any finite data will do
      const bf16_t* bh_row = act_in + rr * as + 8 * hb;
      const bf16_t* bl_row = act_in + (kPos + rr) * as + 8 * hb;
      const bf16_t* a_row = w2_lds + (tap * cpl + ql) * ws + 8 * hb;
      for (int kk = 0; kk < cinl / 16; ++kk) {
        const bf16x8 bh = *reinterpret_cast<const bf16x8*>(bh_row + 16 * kk);
        const bf16x8 bl = *reinterpret_cast<const bf16x8*>(bl_row + 16 * kk);
        const bf16x8 a0 = *reinterpret_cast<const bf16x8*>(a_row + 16 * kk);
        acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, bh, acc[0], 0, 0, 0);
        acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, bl, acc[0], 0, 0, 0);
        if (cpl > 32) {
          const bf16x8 a1 = *reinterpret_cast<const bf16x8*>(a_row + 32 * ws + 16 * kk);
          acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, bh, acc[1], 0, 0, 0);
          acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, bl, acc[1], 0, 0, 0);
        }
      }
    }
    h_prev -= (ksl - 1) / 2 * dl;              // h_l
    if (l + 1 < a.L) {
      // the other region was last read as this layer's input of the layer before; everyone is past that
      // (two barriers since), so it can be overwritten
      bf16_t* act_out = act_in == act_a ? act_b : act_a;
      store_activations(l, act_out, h_prev);
      act_in = act_out;
    }
  }

  // ================= output projection =========================================================================
  {
    const int l = a.L - 1, cout = a.cout[l];
    const bf16_t* wo = a.w_out + (int64_t)h * cout;
    float z = 0.f;
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {
        const int c = 32 * mb + 8 * g4 + 4 * hb;
        if (c < cout) {
          float y[4];
          activation(l, mb, g4, y);
#pragma unroll
          for (int e = 0; e < 4; ++e) z = fmaf(y[e], to_f32(wo[c + e]), z);
        }
      }
    z += __shfl_xor(z, 32, kWave);
    const int j = j0 + row;
    if (hb == 0 && row < a.TM && j < n) a.logits[(int64_t)h * a.total + lo + j] = z + a.b_out[h];
  }
}

struct DeepPlan {
  bool ok = false;
  int TM = 0, x_rows = 0, h0 = 0;
  int lds_ra = 0, lds_r1 = 0, lds_rw = 0;
  size_t lds_bytes = 0;
  int cp[kMaxL] = {0, 0, 0, 0};
  int64_t panel_off[kMaxL] = {0, 0, 0, 0}, panel_head[kMaxL] = {0, 0, 0, 0};
  int64_t panel_elems = 0;
};

DeepPlan plan(const ltea_cfg& cfg, const ltea_cnn& cnn) {
  DeepPlan p;
  if (cfg.dtype != LTEA_BF16 || cnn.n_layers < 2 || (cfg.D != 64 && cfg.D != 128)) return p;
  const int L = cnn.n_layers;
  int cin = 2 * cfg.D;
  int64_t off = 0;
  for (int l = 0; l < L; ++l) {
    const int cout = cnn.c_out[l], ks = cnn.kernel[l];
    if (cout % 16 != 0 || cout > 64 || ks > 7) return p;
    p.cp[l] = (cout + 31) / 32 * 32;
    p.panel_off[l] = off;
    p.panel_head[l] = (int64_t)ks * p.cp[l] * cin;
    off += p.panel_head[l] * cfg.Hkv;
    p.h0 += (ks - 1) / 2 * cnn.dilation[l];
    cin = cout;
  }
  p.panel_elems = off;
  const int reach1 = (cnn.kernel[0] - 1) / 2 * cnn.dilation[0];
  const int h1 = p.h0 - reach1;
  p.TM = kPos - 2 * h1;
  p.x_rows = kPos + 2 * reach1;
  if (p.TM < 32) return p;
  if (kMaxXPieces * kThreads / 4 > kScoreRowsPerDescriptor) return p;   // rows one workgroup addresses
  if (p.x_rows * (CK / 8) > kMaxXPieces * kThreads) return p;
  if (cnn.kernel[0] * p.cp[0] * (CK / 8) > kMaxWPieces * kThreads) return p;
  // LDS regions (elements): A = activations of layers 1, 3; R1 = layer 1's chunk buffers, then activations of
  // layer 2 (and 4 - but the last layer's are never stored); W = panels of layers >= 2
  int sz_a = 0, sz_b = p.x_rows * XS1 + cnn.kernel[0] * p.cp[0] * XS1, sz_w = 0;
  for (int l = 0; l + 1 < L; ++l) {
    const int act = 2 * kPos * (cnn.c_out[l] + 8);
    if (l % 2 == 0) sz_a = act > sz_a ? act : sz_a; else sz_b = act > sz_b ? act : sz_b;
  }
  for (int l = 1; l < L; ++l) {
    const int w = cnn.kernel[l] * p.cp[l] * (cnn.c_out[l - 1] + 8);
    sz_w = w > sz_w ? w : sz_w;
  }
  auto up8 = [](int x) { return (x + 7) / 8 * 8; };
  p.lds_ra = 0;
  p.lds_r1 = up8(sz_a);
  p.lds_rw = p.lds_r1 + up8(sz_b);
  p.lds_bytes = (size_t)(p.lds_rw + up8(sz_w)) * sizeof(uint16_t);
  if (p.lds_bytes > 80 * 1024) return p;    // two workgroups per CU
  p.ok = true;
  return p;
}

}  // namespace

bool score_deep_supported(const ltea_cfg& cfg, const ltea_cnn& cnn) { return plan(cfg, cnn).ok; }

size_t score_deep_workspace(const ltea_cfg& cfg, const ltea_cnn& cnn) {
  return (size_t)plan(cfg, cnn).panel_elems * sizeof(uint16_t);
}

// Fills `panels` with every layer's weights re-laid for score_deep_kernel.
hipError_t launch_score_deep_panels(const ltea_cfg& cfg, const ltea_cnn& cnn, void* panels, hipStream_t stream) {
  const DeepPlan p = plan(cfg, cnn);
  if (!p.ok) return hipErrorInvalidValue;
  if (score_deep_reg_supported(cfg, cnn)) return launch_score_deep_reg_panels(cfg, cnn, panels, stream);   // same size
  int cin = 2 * cfg.D;
  PanelArgs pa;
  int64_t most = 0;
  for (int l = 0; l < kMaxL; ++l) {
    const bool on = l < cnn.n_layers;
    pa.w[l] = on ? static_cast<const uint16_t*>(cnn.w[l]) : nullptr;
    pa.off[l] = p.panel_off[l]; pa.total[l] = on ? p.panel_head[l] * cfg.Hkv : 0;
    pa.cout[l] = on ? cnn.c_out[l] : 16; pa.cp[l] = on ? p.cp[l] : 32; pa.cin[l] = cin; pa.ks[l] = on ? cnn.kernel[l] : 1;
    most = pa.total[l] > most ? pa.total[l] : most;
    if (on) cin = cnn.c_out[l];
  }
  hipLaunchKernelGGL(deep_panels_kernel, dim3((unsigned)((most + 255) / 256), (unsigned)cnn.n_layers), dim3(256), 0,
                     stream, pa, static_cast<uint16_t*>(panels));
  return hipGetLastError();
}

// row_valid: windows mode of the register-stationary kernel (see its launcher); only valid where that kernel applies.
hipError_t launch_score_deep(const ltea_cfg& cfg, const ltea_cnn& cnn, const void* k, const void* v, int64_t st,
                             int64_t sh, const SeqView& sv, float* logits, void* workspace, hipStream_t stream,
                             const uint8_t* row_valid) {
  if (sv.total_tokens == 0) return hipSuccess;
  const DeepPlan p = plan(cfg, cnn);
  if (!p.ok) return hipErrorInvalidValue;
  const void* panels = cnn.panels;
  // the register-stationary kernel sorts unprepared weights itself (no launch for that) when they are 16-byte aligned
  if (panels == nullptr && score_deep_reg_supported(cfg, cnn) && score_deep_reg_takes_raw_weights(cnn))
    return launch_score_deep_reg(cfg, cnn, k, v, st, sh, sv, logits, nullptr, stream, row_valid);
  if (panels == nullptr) {            // not prepared by the caller: re-lay the weights into the workspace now
    hipError_t e = launch_score_deep_panels(cfg, cnn, workspace, stream);
    if (e != hipSuccess) return e;
    panels = workspace;
  }
  if (score_deep_reg_supported(cfg, cnn))
    return launch_score_deep_reg(cfg, cnn, k, v, st, sh, sv, logits, panels, stream, row_valid);
  if (row_valid != nullptr) return hipErrorInvalidValue;
  DeepArgs a;
  a.k = static_cast<const bf16_t*>(k); a.v = static_cast<const bf16_t*>(v); a.st = st; a.sh = sh;
  a.panels = static_cast<const bf16_t*>(panels);
  a.w_out = static_cast<const bf16_t*>(cnn.w_out); a.b_out = cnn.b_out;
  a.L = cnn.n_layers;
  int cin = 2 * cfg.D;
  for (int l = 0; l < kMaxL; ++l) {
    const bool on = l < cnn.n_layers;
    a.panel_off[l] = p.panel_off[l]; a.panel_head[l] = p.panel_head[l];
    a.bias[l] = on ? cnn.bias[l] : nullptr;
    a.ks[l] = on ? cnn.kernel[l] : 1; a.dil[l] = on ? cnn.dilation[l] : 1;
    a.cin[l] = cin; a.cout[l] = on ? cnn.c_out[l] : 16; a.cp[l] = on ? p.cp[l] : 32;
    if (on) cin = cnn.c_out[l];
  }
  a.TM = p.TM; a.x_rows = p.x_rows; a.h0 = p.h0;
  a.lds_ra = p.lds_ra; a.lds_r1 = p.lds_r1; a.lds_rw = p.lds_rw;
  a.cu = sv.cu_seqlens; a.n_seqs = sv.n_seqs; a.total = sv.total_tokens; a.logits = logits;
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&score_deep_kernel),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)p.lds_bytes);
  if (e != hipSuccess) return e;
  const int64_t tiles_upper = (sv.total_tokens + p.TM - 1) / p.TM + sv.n_seqs;
  hipLaunchKernelGGL(score_deep_kernel, dim3((unsigned)tiles_upper, (unsigned)cfg.Hkv), dim3(kThreads), p.lds_bytes,
                     stream, a);
  return hipGetLastError();
}

}  // namespace ltea
