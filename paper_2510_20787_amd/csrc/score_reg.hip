// Scoring CNN of the LTE module (paper Section 3.1.1; Appendix A): single conv layer, bf16, D = 64, with the conv
// weights held in registers.
//
//   z[h][j] = b_out[h] + sum_c w_out[h][c] * Swish( bias[h][c] + sum_{t,m} W[h][c][m][t] * x[j + (t-half)*dil][m] )
// with x = concat(key, value) of the token (128 channels).  As in the LDS-operand kernel the contraction over
// (tap, channel) runs on v_mfma_f32_32x32x16_bf16 as out^T[c, token] = W_t[c, :] . X^T[:, token + shift_t], channels
// (padded to 32) as MFMA rows and 32 tokens per wave as MFMA columns.  What differs:
//   * every wave keeps ALL weight operands of its head (taps x 8 contraction slices x 4 registers: 160 registers
//     for kernel 5, the largest it takes) in registers for the whole workgroup, so only the token operand comes from
//     LDS: half the LDS bytes per MFMA.  The panels are stored in register order ([tap][slice][lane][8]) and reach the
//     registers through LDS, loaded once per workgroup;
//   * token rows go from global memory straight into LDS (buffer_load ... lds, 16 bytes per lane, no staging
//     registers, rows outside the sequence arrive as zeros), keys and values into two arrays of 128-byte rows whose
//     16-byte pieces are XOR-swizzled with the row (a wave instruction fills 1 KB of consecutive LDS, so the
//     permutation is applied to which piece a lane fetches);
//   * four token buffers (one workgroup per CU), one barrier per 128-token tile, loads issued three tiles ahead: with
//     little arithmetic per byte what limits the kernel is how many bytes a CU keeps in flight towards HBM, and three
//     of the four buffers are in flight at any time;
//   * the activation and output projection of a tile are interleaved with the MFMAs of the next one.
// One workgroup = up to 16 consecutive 128-token tiles of one (sequence, KV head) (the host picks the number so that
// the grid is about one workgroup per CU).  Its logits wait in LDS and are stored after the loop, and the epilogue
// constants are loaded before anything else, so that inside the loop the only vector-memory operations in flight are
// the tile loads, which a fixed s_waitcnt vmcnt(N) can then tell apart.
#include "ltea_common.h"
#include "ltea_kernels.h"
#include "score_dma.h"

namespace ltea {
namespace {

constexpr int TM = 128;            // tokens per tile (32 per wave)
constexpr int kThreads = 256;
constexpr int CP = 32;             // channels padded to one MFMA tile
constexpr int kMaxRho = 4;
constexpr int kRowsMax = TM + 2 * kMaxRho;
constexpr int kRowB = 128;         // bytes per row of the key array and of the value array (D = 64)
constexpr int kArrayB = kRowsMax * kRowB;          // one array of one buffer
constexpr int kBufB = 2 * kArrayB;                 // keys then values
constexpr int kBufs = 4;
constexpr int kMaxGroupTiles = 16;
constexpr int kInstrPerArray = (kRowsMax + 7) / 8;                 // wave instructions that cover one array: 17
constexpr int kLdsB = kBufs * kBufB + kMaxGroupTiles * TM * 4;     // 144 KB: the workgroup's logits behind the buffers
constexpr int kLoadsPerWave = 2 * ((kInstrPerArray + 3) / 4);      // per tile and wave, keys + values: 10

// RAW: `panels` is the weight tensor as the caller holds it ([Hkv][C][2D][KS]); the workgroup brings its head's rows
// into LDS and sorts them into register order itself, which saves callers that have not prepared panels a launch.
template <int KS, bool RAW>
__global__ void __launch_bounds__(kThreads, 1)
score_reg_kernel(const bf16_t* __restrict__ k, const bf16_t* __restrict__ v, int64_t st, int64_t sh,
                 const bf16_t* __restrict__ panels, const float* __restrict__ bias,
                 const bf16_t* __restrict__ w_out, const float* __restrict__ b_out, int C, int dil,
                 const int32_t* __restrict__ cu, int n_seqs, int64_t total, float* __restrict__ logits, int group_tiles, int Hkv) {
  constexpr int D = 64, C2 = 2 * D, NSL = C2 / 16;      // 8 contraction slices of 16 channels: 4 of keys, 4 of values
  // four tile buffers, then the workgroup's logits (stored after the loop)
  __shared__ __align__(1024) unsigned char lds[kLdsB];
  const int half = (KS - 1) / 2, rho = half * dil;
  const int tile_rows = TM + 2 * rho;
  // one workgroup per (group of tiles, head), heads fastest: the groups past the last real one (the grid is an upper
  // bound) are then the last to be dispatched and take no CU away from a real one
  const int h = (int)(blockIdx.x % (unsigned)Hkv);
  const int tid = threadIdx.x, lane = tid & 63, ql = lane & 31, hb = lane >> 5;
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
  // The epilogue constants are the only loads left to the compiler; they are issued first and are complete by the time
  // the sequence has been located, so that every later load is a tile or weight transfer counted by hand.
  // accumulator register r of lane half hb is channel 8*(r/4) + 4*hb + r%4 of token ql
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
  float bo = b_out[h];
  int grp, s, n, lo32;
  if (!locate_tile(cu, n_seqs, group_tiles * TM, (int)(blockIdx.x / (unsigned)Hkv), s, grp, lo32, n)) return;
#pragma unroll
  for (int r = 0; r < 16; ++r) asm volatile("" : "+v"(bs[r]), "+v"(wo[r]));
  asm volatile("" : "+v"(bo));
  const int64_t lo = lo32;
  const int g0 = grp * group_tiles * TM;
  int n_tiles = (n - g0 + TM - 1) / TM;
  n_tiles = n_tiles < group_tiles ? n_tiles : group_tiles;

  // ---- global -> LDS -----------------------------------------------------------------------------------------------
  // Descriptors start at the first row this workgroup reads (the sequence start for the first group, whose halo
  // rows then wrap to huge offsets and read as zeros) and end at the last one or at the sequence end.
  const uint32_t row_bytes = (uint32_t)st * 2u;
  const int base_row = g0 > 0 ? g0 - rho : 0;
  const int rows_here = n - base_row < kMaxGroupTiles * TM + 2 * kMaxRho ? n - base_row : kMaxGroupTiles * TM + 2 * kMaxRho;
  const uint32_t span = (uint32_t)(rows_here - 1) * row_bytes + (uint32_t)(D * 2);
  const u32x4 rs_k = make_raw_rsrc(k + (lo + base_row) * st + (int64_t)h * sh, span);
  const u32x4 rs_v = make_raw_rsrc(v + (lo + base_row) * st + (int64_t)h * sh, span);
  const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)lds;
  // A wave instruction covers 8 rows of one array (8 pieces each); instruction j = wv + 4*i covers rows 8j .. 8j+7.
  // Row r keeps piece p in slot p ^ ((r >> 1) & 7): 16 consecutive rows read together then cover all 64 banks.
  // (r >> 1) & 7 for r = 8j + lane/8 is ((lane / 8) >> 1) ^ (4 * (j & 1)), and j & 1 = wv & 1.
  const int ld_piece = (lane & 7) ^ ((((lane >> 3) >> 1) ^ (4 * (wv & 1))) & 7);
  // Every wave issues the same number of loads per tile (kLoadsPerWave), so that one s_waitcnt vmcnt(N) fits all of
  // them: a wave whose turn falls past the last 8-row block fetches the first block once more (same bytes, same place).
  const int n_instr = (tile_rows + 7) / 8;      // per array
  auto issue_tile = [&](int t) {
    const int j0 = g0 + t * TM - rho - base_row;          // first row of the tile relative to the descriptor (may be < 0)
    const int buf = t & (kBufs - 1);
#pragma unroll
    for (int i = 0; i < kLoadsPerWave / 2; ++i) {
      const int jj = wv + 4 * i;
      const int j = jj < n_instr ? jj : wv;
      const uint32_t voff = (uint32_t)(j0 + 8 * j + (lane >> 3)) * row_bytes + (uint32_t)ld_piece * 16u;   // wraps below 0
      const uint32_t dst = lds_base + (uint32_t)(buf * kBufB + j * 1024);
      dma16(rs_k, dst, voff);
      dma16(rs_v, dst + (uint32_t)kArrayB, voff);
    }
  };
  // The head's weights go through LDS as well, once per workgroup: into the fourth tile buffer and the logit area
  // behind it, both idle until the first tile is done.  Either the panels (KS * 8 KB, already in register order
  // [tap][slice][lane][8]), or the caller's rows [c][m][tap]: a row (16 * KS pieces of 16 bytes) is followed by one
  // piece of padding in LDS, so that the 16-byte reads of 16 lanes (16 channels, same column) cover all banks; which
  // piece a lane fetches is computed from where it lands, rows past C and the padding are out of range (zeros).
  constexpr int kRawPieces = 16 * KS;                                // per channel row: 128 inputs x KS taps x 2 bytes
  constexpr int kRawStrideB = (kRawPieces + 1) * 16;
  constexpr int kRawInstr = (CP * (kRawPieces + 1) + 63) / 64;       // wave instructions that cover 32 padded rows
  constexpr int kWeightLoads = RAW ? (kRawInstr + 3) / 4 : 2 * KS;   // per wave
  constexpr int kWeightBase = (kBufs - 1) * kBufB;
  static_assert(kWeightBase + KS * NSL * 1024 <= kLdsB, "weight panels fit behind the third tile buffer");
  static_assert(kWeightBase + kRawInstr * 1024 <= kLdsB, "padded weight rows fit behind the third tile buffer");
  static_assert(kWeightLoads + 3 * kLoadsPerWave <= 63, "loads in flight fit the vmcnt counter");
  issue_tile(0);
  if constexpr (RAW) {
    const u32x4 rs_w = make_raw_rsrc(panels + (int64_t)h * C * C2 * KS, (uint32_t)(C * kRawPieces * 16));
#pragma unroll
    for (int i = 0; i < kWeightLoads; ++i) {
      const int jj = wv + 4 * i;
      const int j = jj < kRawInstr ? jj : wv;           // a turn past the end fetches the wave's first block again
      const int q = 64 * j + lane;                      // piece of the padded LDS image
      const int c = q / (kRawPieces + 1), col = q - c * (kRawPieces + 1);
      const uint32_t voff = col < kRawPieces ? (uint32_t)(c * kRawPieces + col) * 16u : 0x80000000u;
      dma16(rs_w, lds_base + (uint32_t)(kWeightBase + j * 1024), voff);
    }
  } else {
    const u32x4 rs_w = make_raw_rsrc(panels + (int64_t)h * KS * NSL * kWave * 8, (uint32_t)(KS * NSL * 1024));
#pragma unroll
    for (int i = 0; i < kWeightLoads; ++i)
      dma16(rs_w, lds_base + (uint32_t)(kWeightBase + (wv + 4 * i) * 1024), (uint32_t)((wv + 4 * i) * 1024 + lane * 16));
  }
  if (n_tiles > 1) issue_tile(1);
  if (n_tiles > 2) issue_tile(2);
  // first tile and weights: at most the two later tiles may still be in flight
  if (n_tiles > 2) wait_loads_but<2 * kLoadsPerWave>();
  else if (n_tiles > 1) wait_loads_but<kLoadsPerWave>();
  else wait_loads();
  __syncthreads();
  bf16x8 wreg[KS][NSL];
  if constexpr (RAW) {
    // lane (c = ql, hb) owns inputs m = 16*sl + 8*hb .. +7 of every tap: 8 * KS consecutive elements of row c
    typedef unsigned short u16x8 __attribute__((ext_vector_type(8)));
    const unsigned char* wrow = lds + kWeightBase + ql * kRawStrideB + hb * (8 * KS * 2);
#pragma unroll
    for (int sl = 0; sl < NSL; ++sl) {
      u16x8 run[KS];
#pragma unroll
      for (int i = 0; i < KS; ++i) run[i] = *reinterpret_cast<const u16x8*>(wrow + sl * (16 * KS * 2) + 16 * i);
#pragma unroll
      for (int tap = 0; tap < KS; ++tap) {
        u16x8 w;
#pragma unroll
        for (int e = 0; e < 8; ++e) w[e] = run[(e * KS + tap) / 8][(e * KS + tap) % 8];
        wreg[tap][sl] = __builtin_bit_cast(bf16x8, w);
      }
    }
  } else {
#pragma unroll
    for (int tap = 0; tap < KS; ++tap)
#pragma unroll
      for (int sl = 0; sl < NSL; ++sl)
        wreg[tap][sl] = *reinterpret_cast<const bf16x8*>(lds + kWeightBase + (tap * NSL + sl) * 1024 + lane * 16);
  }
  // Pin the weights into their registers here, before the loop's first barrier lets the fourth buffer be refilled.
#pragma unroll
  for (int tap = 0; tap < KS; ++tap)
#pragma unroll
    for (int sl = 0; sl < NSL; ++sl) asm volatile("" : "+v"(wreg[tap][sl]));
  // The tile loop stays rolled: its body is straight-line code of several hundred instructions, and a workgroup that
  // ran eight copies of it once each would spend its time on instruction-cache misses.
  float* zmine = reinterpret_cast<float*>(lds + kBufs * kBufB) + 32 * wv + ql;
  float yprev[16];
#pragma unroll
  for (int r = 0; r < 16; ++r) yprev[r] = 0.f;
#pragma unroll 1
  for (int t = 0; t < n_tiles; ++t) {
    {
      // tile t has landed once at most the loads of the tiles issued after it are still in flight (tiles t+1, t+2)
      if (t + 1 >= n_tiles) wait_loads();
      else if (t + 2 >= n_tiles) wait_loads_but<kLoadsPerWave>();
      else wait_loads_but<2 * kLoadsPerWave>();
      __syncthreads();                 // tile t is in LDS; everyone is done with tile t-1, whose buffer is refilled next
      if (t + 3 < n_tiles) issue_tile(t + 3);
      const unsigned char* buf = lds + (t & (kBufs - 1)) * kBufB;
      f32x16 acc0, acc1, zero;
#pragma unroll
      for (int r = 0; r < 16; ++r) zero[r] = 0.f;
      // The activation and projection of the previous tile (16 values per lane, two transcendentals each) are spread
      // over this tile's MFMAs, one value after every pair: alone they would take as long as the MFMAs again.
      float z = 0.f;
      // token row of this lane for a tap, and where its pieces sit: piece 2*(sl & 3) + hb of the key (sl < 4) or
      // value (sl >= 4) array is in slot (2*(sl & 3) + hb) ^ f, f = (row >> 1) & 7, i.e. at a0 ^ ((sl & 3) << 5)
      auto read_tap = [&](int tap, bf16x8 (&b)[NSL]) {
        const int row = 32 * wv + ql + tap * dil;
        const int f = (row >> 1) & 7;
        const uint32_t a0 = (uint32_t)(row * kRowB + (((f >> 1) << 5) | ((hb ^ (f & 1)) << 4)));
#pragma unroll
        for (int sl = 0; sl < NSL; ++sl)
          b[sl] = *reinterpret_cast<const bf16x8*>(buf + (a0 ^ (uint32_t)((sl & 3) << 5)) + (sl >= 4 ? kArrayB : 0));
      };
      bf16x8 b[2][NSL];                // this tap's operands and the next one's, read one tap ahead
      read_tap(0, b[0]);
#pragma unroll
      for (int tap = 0; tap < KS; ++tap) {
        if (tap + 1 < KS) read_tap(tap + 1, b[(tap + 1) & 1]);
#pragma unroll
        for (int sl = 0; sl < NSL; sl += 2) {
          acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wreg[tap][sl], b[tap & 1][sl], (tap == 0 && sl == 0) ? zero : acc0, 0, 0, 0);
          acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wreg[tap][sl + 1], b[tap & 1][sl + 1], (tap == 0 && sl == 0) ? zero : acc1, 0, 0, 0);
          const int e = tap * (NSL / 2) + sl / 2;
          if (e < 16) z = fmaf(silu_fast(yprev[e]), wo[e], z);
          __builtin_amdgcn_sched_barrier(0);   // keep the interleaving as written
        }
      }
      static_assert(KS * (NSL / 2) >= 12, "pairs to spread the epilogue over");
#pragma unroll
      for (int e = KS * (NSL / 2); e < 16; ++e) z = fmaf(silu_fast(yprev[e]), wo[e], z);
      z = z + __shfl_xor(z, 32, kWave) + bo;
      if (hb == 0 && t > 0) zmine[(t - 1) * TM] = z;
#pragma unroll
      for (int r = 0; r < 16; ++r) yprev[r] = acc0[r] + acc1[r] + bs[r];
    }
  }
  {
    float z = 0.f;
#pragma unroll
    for (int r = 0; r < 16; ++r) z = fmaf(silu_fast(yprev[r]), wo[r], z);
    z = z + __shfl_xor(z, 32, kWave) + bo;
    if (hb == 0) zmine[(n_tiles - 1) * TM] = z;
  }
  // every lane stores what it put there itself: no barrier
  for (int t = 0; t < n_tiles; ++t) {
    const int j = g0 + t * TM + 32 * wv + ql;
    if (hb == 0 && j < n) logits[(int64_t)h * total + lo + j] = zmine[t * TM];
  }
}

// panels[h][tap][sl][lane][e] = W[h][c][m][tap], c = lane % 32 (0 beyond C), m = 16*sl + 8*(lane / 32) + e
__global__ void __launch_bounds__(256)
score_reg_panels_kernel(const uint16_t* __restrict__ W, uint16_t* __restrict__ panels, int C, int C2, int ks,
                        int64_t total) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= total) return;
  const int e = (int)(idx & 7);
  const int ln = (int)((idx >> 3) & 63);
  int64_t r = idx >> 9;
  const int nsl = C2 / 16;
  const int sl = (int)(r % nsl); r /= nsl;
  const int tap = (int)(r % ks);
  const int64_t h = r / ks;
  const int c = ln & 31, m = 16 * sl + 8 * (ln >> 5) + e;
  panels[idx] = c < C ? W[((h * C + c) * C2 + m) * ks + tap] : (uint16_t)0;
}

template <int KS, bool RAW>
hipError_t run(const ltea_cfg& cfg, const ltea_cnn& cnn, const void* k, const void* v, int64_t st, int64_t sh,
               const SeqView& sv, float* logits, const void* weights, hipStream_t stream) {
  const int gt = pick_group_tiles(sv, cfg.Hkv, TM, kMaxGroupTiles);
  const int64_t groups_upper = (sv.total_tokens + gt * TM - 1) / (gt * TM) + sv.n_seqs;
  hipLaunchKernelGGL((score_reg_kernel<KS, RAW>), dim3((unsigned)(groups_upper * cfg.Hkv)), dim3(kThreads), 0, stream,
                     static_cast<const bf16_t*>(k), static_cast<const bf16_t*>(v), st, sh,
                     static_cast<const bf16_t*>(weights), cnn.bias[0], static_cast<const bf16_t*>(cnn.w_out), cnn.b_out,
                     cnn.c_out[0], cnn.dilation[0], sv.cu_seqlens, sv.n_seqs, sv.total_tokens, logits, gt, cfg.Hkv);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_score_reg_panels(const ltea_cfg& cfg, const ltea_cnn& cnn, void* panels, hipStream_t stream) {
  const int ks = cnn.kernel[0], C2 = 2 * cfg.D;
  const int64_t panel_elems = (int64_t)cfg.Hkv * ks * CP * C2;
  hipLaunchKernelGGL(score_reg_panels_kernel, dim3((unsigned)((panel_elems + 255) / 256)), dim3(256), 0, stream,
                     static_cast<const uint16_t*>(cnn.w[0]), static_cast<uint16_t*>(panels), cnn.c_out[0], C2, ks,
                     panel_elems);
  return hipGetLastError();
}

// Same weight panels ([Hkv][taps][32][2D], channels zero-padded to 32) and same dispatch conditions as the LDS-operand
// kernel, restricted to D = 64 and kernel sizes whose operands fit the register file.
bool score_reg_supported(const ltea_cfg& cfg, const ltea_cnn& cnn) {
  if (cfg.dtype != LTEA_BF16 || cnn.n_layers != 1 || cnn.c_out[0] > CP || cfg.D != 64) return false;
  const int ks = cnn.kernel[0];
  if (ks != 3 && ks != 5) return false;    // kernel 7 would need 224 registers for the weights alone
  static_assert(kMaxGroupTiles * TM + 2 * kMaxRho + 16 <= kScoreRowsPerDescriptor, "rows one workgroup addresses");
  return (ks - 1) / 2 * cnn.dilation[0] <= kMaxRho;
}

bool score_reg_takes_raw_weights(const ltea_cnn& cnn) { return (reinterpret_cast<uintptr_t>(cnn.w[0]) & 15u) == 0; }

hipError_t launch_score_reg(const ltea_cfg& cfg, const ltea_cnn& cnn, const void* k, const void* v, int64_t st,
                            int64_t sh, const SeqView& sv, float* logits, const void* panels, hipStream_t stream) {
  if (sv.total_tokens == 0) return hipSuccess;
  if (panels == nullptr) {   // the kernel sorts the caller's weight rows into register order itself
    if (!score_reg_takes_raw_weights(cnn)) return hipErrorInvalidValue;
    return cnn.kernel[0] == 3 ? run<3, true>(cfg, cnn, k, v, st, sh, sv, logits, cnn.w[0], stream)
                              : run<5, true>(cfg, cnn, k, v, st, sh, sv, logits, cnn.w[0], stream);
  }
  return cnn.kernel[0] == 3 ? run<3, false>(cfg, cnn, k, v, st, sh, sv, logits, panels, stream)
                            : run<5, false>(cfg, cnn, k, v, st, sh, sv, logits, panels, stream);
}

}  // namespace ltea
