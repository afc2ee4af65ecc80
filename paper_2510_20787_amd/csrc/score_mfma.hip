// Scoring CNN of the LTE module (paper Section 3.1.1; Appendix A): fused single-layer bf16 path on MFMA.
//
//   z[h][j] = b_out[h] + sum_c w_out[h][c] * Swish( bias[h][c] + sum_{t,m} W[h][c][m][t] * x[j + (t-half)*dil][m] )
// with x = concat(key, value) of the token (2*D channels).  The contraction over (tap, channel) is a small
// GEMM per head: out^T[c, token] = W_t[c, :] . X^T[:, token + shift_t], run on v_mfma_f32_32x32x16_bf16 with
// the (zero-padded to 32) channels as MFMA rows and 32 tokens per wave as MFMA columns.  In the accumulator
// layout one lane owns one token, so bias, Swish and the output projection are per-lane work on the 16
// channel values it holds plus one exchange with the lane holding the other 16.
//
// Two launches:
//   score_weight_panels_kernel  re-lays the weights [Hkv][C][2D][k] once per call as tap-major panels
//                               [Hkv][k][32][2D] (channels zero-padded to 32) in the workspace, so that the main
//                               kernel can fetch a panel with coalesced 16-byte loads;
//   score_mfma_kernel           one workgroup = 4 consecutive 128-token tiles of one (sequence, KV head).  Input
//                               channels are processed in chunks of 128 (D = 64: keys and values together;
//                               D = 128: keys, then values): all taps' weight panels of the chunk are staged in
//                               LDS once and reused for the four tiles (one accumulator set per tile); each
//                               tile's rows with their halo of half*dil rows (zeros outside the sequence) are
//                               fetched into registers while the previous tile is being multiplied and then
//                               stored to LDS in 16-byte pieces.  Rows are padded by 16 bytes, which makes the
//                               16-lane groups of every ds_read_b128 hit 64 distinct banks.
#include "ltea_common.h"
#include "ltea_kernels.h"

namespace ltea {
namespace {

constexpr int TM = 128;       // tokens per workgroup
constexpr int kThreads = 256;
constexpr int CP = 32;        // channels padded to one MFMA tile
constexpr int CH = 128;       // input channels per chunk
constexpr int XS = CH + 8;    // LDS row stride (elements) of the token tile and of the weight panel
constexpr int NT = 4;         // consecutive token tiles per workgroup (weights staged once for all of them)
constexpr int kMaxRho = 4;    // largest half receptive field the token tile is sized for
constexpr int kTileRows = TM + 2 * kMaxRho;   // LDS rows of the token tile

// panels[h][tap][c][m] = W[h][c][m][tap] for c < C, 0 for C <= c < 32
__global__ void __launch_bounds__(256)
score_weight_panels_kernel(const uint16_t* __restrict__ W, uint16_t* __restrict__ panels, int C, int C2, int ks,
                           int64_t total) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;   // over [Hkv][ks][32][C2]
  if (idx >= total) return;
  const int m = (int)(idx % C2);
  int64_t r = idx / C2;
  const int c = (int)(r % CP); r /= CP;
  const int tap = (int)(r % ks);
  const int64_t h = r / ks;
  panels[idx] = c < C ? W[((h * C + c) * C2 + m) * ks + tap] : (uint16_t)0;
}

template <int D>
__global__ void __launch_bounds__(kThreads)
score_mfma_kernel(const bf16_t* __restrict__ k, const bf16_t* __restrict__ v, int64_t st, int64_t sh,
                  const bf16_t* __restrict__ panels, const float* __restrict__ bias,
                  const bf16_t* __restrict__ w_out, const float* __restrict__ b_out, int C, int ks, int dil,
                  const int32_t* __restrict__ cu, int n_seqs, int groups_upper, int64_t total,
                  float* __restrict__ logits) {
  constexpr int C2 = 2 * D;        // input channels
  constexpr int NCH = C2 / CH;     // chunks
  constexpr int PPR = CH / 8;      // 16-byte pieces per chunk row (16)
  constexpr int RPP = kThreads / PPR;   // token rows per staging pass (16)
  constexpr int XREG = (TM + 2 * kMaxRho + RPP - 1) / RPP;   // staging passes (registers) per tile
  extern __shared__ __align__(16) unsigned char smem[];
  const int half = (ks - 1) / 2, rho = half * dil;
  const int tile_rows = TM + 2 * rho;              // rows of the token tile actually used (at most kTileRows)
  bf16_t* x_lds = reinterpret_cast<bf16_t*>(smem);
  bf16_t* w_lds = x_lds + (size_t)tile_rows * XS;  // ks panels of CP x XS (all taps of the current chunk)

  const int h = blockIdx.y;
  int grp, s, n, lo32;
  if (!locate_tile(cu, n_seqs, NT * TM, blockIdx.x, s, grp, lo32, n)) return;
  const int64_t lo = lo32;
  const int g0 = grp * NT * TM;                      // first token of this workgroup's NT tiles
  int n_tiles = (n - g0 + TM - 1) / TM;
  n_tiles = n_tiles < NT ? n_tiles : NT;
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, ql = lane & 31, hb = lane >> 5;

  const bf16_t* ph = panels + (int64_t)h * ks * CP * C2;
  // all taps' panels of one chunk -> LDS: 512 coalesced 16-byte pieces per tap, two per thread, no conditions
  auto stage_panels = [&](int chunk) {
    const int pm = (tid % (CH / 8)) * 8, c0 = tid / (CH / 8);           // channels c0 and c0 + 16
    const bf16_t* src = ph + (int64_t)c0 * C2 + chunk * CH + pm;
    bf16_t* dst = w_lds + (size_t)c0 * XS + pm;
    for (int tap0 = 0; tap0 < ks; tap0 += 4) {
      u32x4 w[4][2];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int tap = tap0 + u < ks ? tap0 + u : ks - 1;                // clamp: the extra copies are harmless
        w[u][0] = *reinterpret_cast<const u32x4*>(src + (int64_t)tap * CP * C2);
        w[u][1] = *reinterpret_cast<const u32x4*>(src + (int64_t)tap * CP * C2 + 16 * C2);
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int tap = tap0 + u < ks ? tap0 + u : ks - 1;
        *reinterpret_cast<u32x4*>(dst + (size_t)tap * CP * XS) = w[u][0];
        *reinterpret_cast<u32x4*>(dst + (size_t)tap * CP * XS + 16 * XS) = w[u][1];
      }
    }
  };
  // Token tile of one chunk with halo: global -> registers (issued early), registers -> LDS (after the MFMAs).
  // Buffer loads: rows before the sequence start or past its end are outside the descriptor and read as zeros,
  // so the loads carry no conditions and are issued back to back.  For D = 64 a chunk row is 8 key pieces followed
  // by 8 value pieces; waves 0-1 fetch the key halves and waves 2-3 the value halves (one descriptor per wave).
  constexpr int HT = D == 64 ? kThreads / 2 : kThreads;   // threads cooperating on one tensor's part of the rows
  constexpr int PPH = D == 64 ? 8 : 16;                   // 16-byte pieces of that part per row
  const int t_in = tid % HT, piece = t_in % PPH, r_in = t_in / PPH;   // 16 rows per pass either way
  const bool v_wave = D == 64 && __builtin_amdgcn_readfirstlane(tid / HT) == 1;
  // The descriptors start at the first row this workgroup reads (the sequence start for the first group, whose
  // halo rows then wrap to huge offsets) and end at the last one or at the sequence end, so that 32-bit byte
  // offsets only ever span one group of tiles however long the sequence is.
  const uint32_t row_bytes = (uint32_t)st * 2u;
  const int base_row = g0 > 0 ? g0 - rho : 0;
  const int rows_here = n - base_row < NT * TM + 2 * kMaxRho ? n - base_row : NT * TM + 2 * kMaxRho;
  const uint32_t seq_bytes = (uint32_t)(rows_here - 1) * row_bytes + (uint32_t)(D * 2);
  const int64_t base_el = (lo + base_row) * st + (int64_t)h * sh;
  const auto rs_k = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t*>(k + base_el), 0, seq_bytes, 0x00020000);
  const auto rs_v = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t*>(v + base_el), 0, seq_bytes, 0x00020000);
  const int lds_col = (v_wave ? D : 0) + piece * 8;
  u32x4 xreg[XREG];
  auto load_tokens = [&](int chunk, int tile) {
    const bool is_v = D == 64 ? v_wave : chunk == 1;
    const int j0 = g0 + tile * TM;
    const uint32_t off0 = (uint32_t)(j0 - rho + r_in - base_row) * row_bytes + (uint32_t)piece * 16u;   // wraps for rows < 0
#pragma unroll
    for (int i = 0; i < XREG; ++i) {
      const uint32_t off = off0 + (uint32_t)(i * RPP) * row_bytes;
      xreg[i] = is_v ? __builtin_amdgcn_raw_buffer_load_b128(rs_v, off, 0, 0)
                     : __builtin_amdgcn_raw_buffer_load_b128(rs_k, off, 0, 0);
    }
  };
  auto store_tokens = [&]() {
#pragma unroll
    for (int i = 0; i < XREG; ++i)
      if (r_in + i * RPP < tile_rows)   // the token tile ends where the weight panels begin
        *reinterpret_cast<u32x4*>(&x_lds[(r_in + i * RPP) * XS + lds_col]) = xreg[i];
  };

  f32x16 acc[NT];
#pragma unroll
  for (int t = 0; t < NT; ++t)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[t][r] = 0.f;

  load_tokens(0, 0);
  for (int chunk = 0; chunk < NCH; ++chunk) {
    __syncthreads();                 // previous chunk's panels and token tile are no longer read
    stage_panels(chunk);
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      if (t < n_tiles) {             // uniform
        if (t > 0) __syncthreads();  // previous tile's rows are no longer read
        store_tokens();
        __syncthreads();
        // prefetch the next token tile (next tile of this chunk, or first tile of the next chunk)
        if (t + 1 < n_tiles) load_tokens(chunk, t + 1);
        else if (chunk + 1 < NCH) load_tokens(chunk + 1, 0);
        for (int tap = 0; tap < ks; ++tap) {
          const bf16_t* a_row = w_lds + (size_t)(tap * CP + ql) * XS + 8 * hb;                // channel ql
          const bf16_t* b_row = x_lds + (size_t)(32 * wv + ql + tap * dil) * XS + 8 * hb;     // token, shifted
#pragma unroll
          for (int mc = 0; mc < CH / 16; ++mc) {
            const bf16x8 a = *reinterpret_cast<const bf16x8*>(a_row + 16 * mc);
            const bf16x8 b = *reinterpret_cast<const bf16x8*>(b_row + 16 * mc);
            acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[t], 0, 0, 0);
          }
          // Issue order inside one tap: operand reads run three MFMAs ahead of their use, so that LDS latency is
          // covered by matrix work instead of being waited for before every MFMA.
          __builtin_amdgcn_sched_group_barrier(0x100, 6, 0);
#pragma unroll
          for (int i = 0; i < CH / 16 - 3; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
          }
          __builtin_amdgcn_sched_group_barrier(0x008, 3, 0);
        }
      }
    }
  }

  // ---- epilogue: accumulator register r of lane half hb is channel 8*(r/4) + 4*hb + r%4 of token ql ----------
  float bs[16], wo[16];
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    const int c = 8 * (r / 4) + 4 * hb + (r % 4);
    const int cc = c < C ? c : C - 1;            // unconditional loads (no branch per element), then select
    const float b_ld = bias[h * C + cc];
    const float w_ld = to_f32(w_out[h * C + cc]);
    bs[r] = c < C ? b_ld : 0.f;
    wo[r] = c < C ? w_ld : 0.f;
  }
  const float bo = b_out[h];
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    if (t < n_tiles) {
      float z = 0.f;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float y = acc[t][r] + bs[r];
        z = fmaf(y * __frcp_rn(1.0f + __expf(-y)), wo[r], z);
      }
      z += __shfl_xor(z, 32, kWave);
      const int j = g0 + t * TM + 32 * wv + ql;
      if (hb == 0 && j < n) logits[(int64_t)h * total + lo + j] = z + bo;
    }
  }
}

// Token tile sized by the actual reach: 79.4 KB for kernel 5 / dilation 1, so that two workgroups share a CU.
size_t lds_bytes(int ks, int dil) {
  const int rho = (ks - 1) / 2 * dil;
  return ((size_t)(TM + 2 * rho) + (size_t)ks * CP) * XS * sizeof(uint16_t);
}

template <int D>
hipError_t run(const ltea_cfg& cfg, const ltea_cnn& cnn, const void* k, const void* v, int64_t st, int64_t sh,
               const SeqView& sv, float* logits, void* workspace, hipStream_t stream) {
  const int ks = cnn.kernel[0];
  const void* panels = cnn.panels;
  hipError_t e = hipSuccess;
  // the register-stationary kernel sorts unprepared weights itself (no launch for that) when they are 16-byte aligned
  if (panels == nullptr && score_reg_supported(cfg, cnn) && score_reg_takes_raw_weights(cnn))
    return launch_score_reg(cfg, cnn, k, v, st, sh, sv, logits, nullptr, stream);
  if (panels == nullptr) {            // not prepared by the caller: re-lay the weights into the workspace now
    e = launch_score_mfma_panels(cfg, cnn, workspace, stream);
    if (e != hipSuccess) return e;
    panels = workspace;
  }
  if (score_reg_supported(cfg, cnn)) return launch_score_reg(cfg, cnn, k, v, st, sh, sv, logits, panels, stream);
  const size_t lds = lds_bytes(ks, cnn.dilation[0]);
  e = hipFuncSetAttribute(reinterpret_cast<const void*>(&score_mfma_kernel<D>),
                          hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  if (e != hipSuccess) return e;
  const int64_t groups_upper = (sv.total_tokens + NT * TM - 1) / (NT * TM) + sv.n_seqs;
  hipLaunchKernelGGL(score_mfma_kernel<D>, dim3((unsigned)groups_upper, (unsigned)cfg.Hkv), dim3(kThreads), lds, stream,
                     static_cast<const bf16_t*>(k), static_cast<const bf16_t*>(v), st, sh,
                     static_cast<const bf16_t*>(panels), cnn.bias[0], static_cast<const bf16_t*>(cnn.w_out),
                     cnn.b_out, cnn.c_out[0], ks, cnn.dilation[0], sv.cu_seqlens, sv.n_seqs, (int)groups_upper,
                     sv.total_tokens, logits);
  return hipGetLastError();
}

}  // namespace

bool score_mfma_supported(const ltea_cfg& cfg, const ltea_cnn& cnn) {
  if (cfg.dtype != LTEA_BF16 || cnn.n_layers != 1 || cnn.c_out[0] > CP) return false;
  if (cfg.D != 64 && cfg.D != 128) return false;
  if ((cnn.kernel[0] - 1) / 2 * cnn.dilation[0] > kMaxRho) return false;
  static_assert(NT * TM + 2 * kMaxRho + 16 <= kScoreRowsPerDescriptor, "rows one workgroup addresses");
  return lds_bytes(cnn.kernel[0], cnn.dilation[0]) <= 150 * 1024;
}

hipError_t launch_score_mfma_panels(const ltea_cfg& cfg, const ltea_cnn& cnn, void* panels, hipStream_t stream) {
  if (score_reg_supported(cfg, cnn)) return launch_score_reg_panels(cfg, cnn, panels, stream);   // its own order, same size
  const int ks = cnn.kernel[0], C2 = 2 * cfg.D;
  const int64_t panel_elems = (int64_t)cfg.Hkv * ks * CP * C2;
  hipLaunchKernelGGL(score_weight_panels_kernel, dim3((unsigned)((panel_elems + 255) / 256)), dim3(256), 0, stream,
                     static_cast<const uint16_t*>(cnn.w[0]), static_cast<uint16_t*>(panels), cnn.c_out[0], C2, ks,
                     panel_elems);
  return hipGetLastError();
}

size_t score_mfma_workspace(const ltea_cfg& cfg, const ltea_cnn& cnn) {
  return (size_t)cfg.Hkv * cnn.kernel[0] * CP * 2 * cfg.D * sizeof(uint16_t);
}

hipError_t launch_score_mfma(const ltea_cfg& cfg, const ltea_cnn& cnn, const void* k, const void* v, int64_t st,
                             int64_t sh, const SeqView& sv, float* logits, void* workspace, hipStream_t stream) {
  if (sv.total_tokens == 0) return hipSuccess;
  return cfg.D == 64 ? run<64>(cfg, cnn, k, v, st, sh, sv, logits, workspace, stream)
                     : run<128>(cfg, cnn, k, v, st, sh, sv, logits, workspace, stream);
}

}  // namespace ltea
