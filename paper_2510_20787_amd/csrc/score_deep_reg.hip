// Scoring CNN of the LTE module in the paper's own shape (Section 3.1.1, Appendix A: three k = 3 dilated layers,
// 2D = 128 -> 64 -> 32 -> 16 channels, then a linear projection to one logit), bf16, with every layer's weights held in
// registers.
//
//   a_0[j] = concat(key_j, value_j);  a_l[j][c] = Swish( bias_l[c] + sum_{t,m} W_l[c][m][t] * a_{l-1}[j + (t-1)*dil_l][m] )
//   z[j] = b_out + sum_c w_out[c] * a_3[j][c];   activations of positions outside the sequence are zero at every layer.
//
// Same arithmetic as the general multi-layer kernel (output channels as MFMA rows, 32 positions per wave as MFMA
// columns, every layer computes 128 consecutive positions anchored so that a later layer finds its inputs among them,
// intermediate activations in LDS as hi + lo bf16 pairs, each multiplied by the bf16 weights in its own MFMA).  What
// differs is where the operands live and how a workgroup is fed:
//   * all 66 KB of a head's weights (48 + 12 + 6 operand blocks of 4 registers) stay in each wave's registers for the
//     whole workgroup; they arrive once, through LDS, in register order;
//   * token rows go from global memory straight into LDS (buffer_load ... lds), keys and values into two arrays of
//     128-byte rows with XOR-swizzled 16-byte pieces, three tile buffers, loads issued up to three tiles ahead: a
//     tile's buffer is free again as soon as its first layer is done;
//   * one workgroup per CU takes a run of consecutive tiles of one (sequence, KV head); its logits wait in LDS and are
//     stored after the loop, and the few constants (biases, projection) are loaded before anything else, so that inside
//     the loop the only vector-memory operations in flight are the tile loads, which a fixed s_waitcnt vmcnt(N) counts.
#include "ltea_common.h"
#include "ltea_kernels.h"
#include "score_dma.h"

namespace ltea {
namespace {

constexpr int kPos = 128;          // positions every layer computes per tile (32 per wave)
constexpr int kThreads = 256;
constexpr int C1 = 64, C2 = 32, C3 = 16;          // output channels of the three layers
constexpr int kMaxD1 = 4;                         // first layer's dilation: a tile has 128 + 2*d1 <= 136 input rows
constexpr int kRowsMax = kPos + 2 * kMaxD1;
constexpr int kRowB = 128;                        // bytes per row of the key array and of the value array (D = 64)
constexpr int kArrayB = kRowsMax * kRowB;
constexpr int kBufB = 2 * kArrayB;                // keys then values
constexpr int kBufs = 3;
constexpr int kActAB = 2 * kPos * 2 * C1;         // layer 1's output: hi array then lo array of 128-byte rows
constexpr int kActBB = 2 * kPos * 2 * C2;         // layer 2's output: hi array then lo array of 64-byte rows
constexpr int kConsts = C1 + C2 + C3 + C3;        // bias1, bias2, bias3, w_out as floats
constexpr int kMaxGroupTiles = 16;
constexpr int kOffActA = kBufs * kBufB;
constexpr int kOffActB = kOffActA + kActAB;
constexpr int kOffConst = kOffActB + kActBB;
constexpr int kOffZ = kOffConst + kConsts * 4;
constexpr int kOffValid = kOffZ + kMaxGroupTiles * kPos * 4;
constexpr int kMostRows = kMaxGroupTiles * kPos + 2 * kMaxD1;      // rows one workgroup's descriptor spans at most
constexpr int kValidWords = (kMostRows + 63) / 64 * 2;             // one bit per row
constexpr int kLdsB = kOffValid + kValidWords * 4;
static_assert(kLdsB <= 160 * 1024, "one workgroup's LDS");
constexpr int kInstrPerArray = (kRowsMax + 7) / 8;                 // wave instructions that cover one array: 17
constexpr int kLoadsPerWave = 2 * ((kInstrPerArray + 3) / 4);      // per tile and wave, keys + values: 10
constexpr int kBlocks1 = 3 * 8 * 2, kBlocks2 = 3 * 4, kBlocks3 = 3 * 2;   // 1 KB operand blocks: [tap][slice][(mb)]
constexpr int kBlocks = kBlocks1 + kBlocks2 + kBlocks3;                   // 66 per head
constexpr int kWeightLoadsPerWave = (kBlocks + 3) / 4;
static_assert(kBlocks * 1024 <= 2 * kBufB, "the weights pass through the second and third tile buffers");
// Weights that were not re-laid beforehand come as the caller's rows [c][m][tap] (16-byte pieces: 3 * c_in / 8 per row)
// and are sorted into operands by the workgroup.  In LDS every row is followed by one piece of padding, which makes the
// row strides 196, 100 and 52 words: the 16-byte reads of 16 lanes (16 channels, same column) then cover all banks.
// Each tensor's image is rounded up to whole wave instructions (1 KB); the third layer brings its 16 real rows only.
constexpr int kRawP1 = 3 * 2 * 64 / 8, kRawP2 = 3 * C1 / 8, kRawP3 = 3 * C2 / 8;        // pieces per row: 48, 24, 12
constexpr int kRawI1 = (C1 * (kRawP1 + 1) + 63) / 64, kRawI2 = (C2 * (kRawP2 + 1) + 63) / 64,
              kRawI3 = (C3 * (kRawP3 + 1) + 63) / 64;                                   // wave instructions: 49, 13, 4
static_assert(kRawI1 + kRawI2 + kRawI3 <= kBlocks, "same number of weight loads per wave either way");
static_assert(kLoadsPerWave + kWeightLoadsPerWave <= 63 && 2 * kLoadsPerWave <= 63, "loads in flight fit vmcnt");

struct DeepRegArgs {
  const bf16_t* k; const bf16_t* v; int64_t st, sh;
  const bf16_t* panels;                       // [Hkv][66][64 lanes][8], or null: the three tensors below as the caller holds them
  const bf16_t* w1; const bf16_t* w2; const bf16_t* w3;   // [Hkv][c_out][c_in][3]
  const float* bias1; const float* bias2; const float* bias3; const bf16_t* w_out; const float* b_out;
  int d1, d2, d3;
  const int32_t* cu; int n_seqs; int64_t total; float* logits; int group_tiles, Hkv;
  const uint8_t* row_valid;   // optional [total]: 0 marks a row that is padding between independent short windows
};

__global__ void __launch_bounds__(kThreads, 1)
score_deep_reg_kernel(const DeepRegArgs a) {
  __shared__ __align__(1024) unsigned char lds[kLdsB];
  const int h = (int)(blockIdx.x % (unsigned)a.Hkv);       // heads fastest: the groups past the last real one come last
  const int tid = threadIdx.x, lane = tid & 63, ql = lane & 31, hb = lane >> 5;
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int row = 32 * wv + ql;                            // this lane's position index inside every layer's 128

  // The constants are the only loads left to the compiler; they are issued first and are complete by the time the
  // sequence has been located.
  float cval = 0.f;
  if (tid < C1) cval = a.bias1[h * C1 + tid];
  else if (tid < C1 + C2) cval = a.bias2[h * C2 + tid - C1];
  else if (tid < C1 + C2 + C3) cval = a.bias3[h * C3 + tid - C1 - C2];
  else if (tid < kConsts) cval = to_f32(a.w_out[h * C3 + tid - C1 - C2 - C3]);
  float bo = a.b_out[h];
  const int h1 = a.d2 + a.d3, h0 = a.d1 + h1;              // half receptive fields behind layer 1 / of the stack
  const int TMv = kPos - 2 * h1;                           // positions of a tile whose logits are exact
  int grp, s, n, lo32;
  if (!locate_tile(a.cu, a.n_seqs, a.group_tiles * TMv, (int)(blockIdx.x / (unsigned)a.Hkv), s, grp, lo32, n)) return;
  asm volatile("" : "+v"(cval), "+v"(bo));
  float* consts = reinterpret_cast<float*>(lds + kOffConst);
  if (tid < kConsts) consts[tid] = cval;                   // read after the barriers below
  const int64_t lo = lo32;
  const int g0 = grp * a.group_tiles * TMv;
  int n_tiles = (n - g0 + TMv - 1) / TMv;
  n_tiles = n_tiles < a.group_tiles ? n_tiles : a.group_tiles;

  // ---- global -> LDS -----------------------------------------------------------------------------------------------
  // Descriptors start at the first row this workgroup reads (the sequence start for the first group, whose halo
  // rows then wrap to huge offsets and read as zeros) and end at the last one or at the sequence end.
  const uint32_t row_bytes = (uint32_t)a.st * 2u;
  const int base_row = g0 > 0 ? g0 - h0 : 0;
  const int rows_here = n - base_row < kMostRows ? n - base_row : kMostRows;
  // Windows mode (decode: many independent short windows packed with zero rows between them): one bit per row of this
  // workgroup's range says whether it is a real token; activations of the others are forced to zero at every layer,
  // exactly as outside a sequence.  Loaded now, with ordinary loads, before any tile load is in flight.
  uint32_t* valid_bits = reinterpret_cast<uint32_t*>(lds + kOffValid);
  if (a.row_valid != nullptr) {
    for (int r0 = 64 * wv; r0 < rows_here; r0 += 64 * 4) {
      const int r = base_row + r0 + lane;
      const uint8_t f = r < n ? a.row_valid[lo + r] : (uint8_t)0;
      const unsigned long long m = __builtin_amdgcn_ballot_w64(f != 0);
      if (lane == 0) { valid_bits[r0 >> 5] = (uint32_t)m; valid_bits[(r0 >> 5) + 1] = (uint32_t)(m >> 32); }
    }
  }
  const uint32_t span = (uint32_t)(rows_here - 1) * row_bytes + (uint32_t)kRowB;
  const u32x4 rs_k = make_raw_rsrc(a.k + (lo + base_row) * a.st + (int64_t)h * a.sh, span);
  const u32x4 rs_v = make_raw_rsrc(a.v + (lo + base_row) * a.st + (int64_t)h * a.sh, span);
  const u32x4 rs_w = make_raw_rsrc(a.panels + (int64_t)h * kBlocks * 512, (uint32_t)(kBlocks * 1024));
  const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)lds;
  // A wave instruction covers 8 rows of one array (8 pieces each); instruction j = wv + 4*i covers rows 8j .. 8j+7.
  // Row r keeps piece p in slot p ^ ((r >> 1) & 7): 16 consecutive rows read together then cover all 64 banks.
  // (r >> 1) & 7 for r = 8j + lane/8 is ((lane / 8) >> 1) ^ (4 * (j & 1)), and j & 1 = wv & 1.
  const int ld_piece = (lane & 7) ^ ((((lane >> 3) >> 1) ^ (4 * (wv & 1))) & 7);
  // Every wave issues the same number of loads per tile, so that one s_waitcnt vmcnt(N) fits all of them: a wave whose
  // turn falls past the last 8-row block fetches its first block once more (same bytes, same place).
  const int n_instr = (kPos + 2 * a.d1 + 7) / 8;
  auto issue_tile = [&](int t, int buf) {
    const int j0 = g0 + t * TMv - h0 - base_row;          // first row of the tile relative to the descriptor (may be < 0)
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
  issue_tile(0, 0);
  const bool raw = a.panels == nullptr;
  if (!raw) {
#pragma unroll
    for (int i = 0; i < kWeightLoadsPerWave; ++i) {
      const int bb = wv + 4 * i;
      const int b = bb < kBlocks ? bb : wv;
      dma16(rs_w, lds_base + (uint32_t)(kBufB + b * 1024), (uint32_t)(b * 1024 + lane * 16));
    }
  } else {
    // instruction b fills pieces 64*b .. 64*b+63 of the padded images [layer 1 | layer 2 | layer 3]; which piece of
    // which row a lane fetches follows from where it lands; padding and rows past the tensor are out of range (zeros)
    const u32x4 rs_1 = make_raw_rsrc(a.w1 + (int64_t)h * C1 * 2 * 64 * 3, (uint32_t)(C1 * kRawP1 * 16));
    const u32x4 rs_2 = make_raw_rsrc(a.w2 + (int64_t)h * C2 * C1 * 3, (uint32_t)(C2 * kRawP2 * 16));
    const u32x4 rs_3 = make_raw_rsrc(a.w3 + (int64_t)h * C3 * C2 * 3, (uint32_t)(C3 * kRawP3 * 16));
#pragma unroll
    for (int i = 0; i < kWeightLoadsPerWave; ++i) {
      const int bb = wv + 4 * i;
      const int b = bb < kRawI1 + kRawI2 + kRawI3 ? bb : wv;
      const int layer = b < kRawI1 ? 0 : (b < kRawI1 + kRawI2 ? 1 : 2);
      const int q = 64 * (b - (layer == 0 ? 0 : (layer == 1 ? kRawI1 : kRawI1 + kRawI2))) + lane;
      const int pr = layer == 0 ? kRawP1 : (layer == 1 ? kRawP2 : kRawP3);
      const int c = q / (pr + 1), col = q - c * (pr + 1);
      const uint32_t voff = col < pr ? (uint32_t)(c * pr + col) * 16u : 0x80000000u;
      const u32x4 rs = layer == 0 ? rs_1 : (layer == 1 ? rs_2 : rs_3);
      dma16(rs, lds_base + (uint32_t)(kBufB + b * 1024), voff);
    }
  }
  wait_loads();
  __syncthreads();

  // ---- weights -> registers: A operand of (tap, slice[, channel block]): output channel ql (+ 32 per block), input
  // channels 16*slice + 8*hb .. +7 --------------------------------------------------------------------------------
  bf16x8 w1[3][8][2], w2[3][4], w3[3][2];
  if (raw) {
    // a lane's inputs 16*slice + 8*hb .. +7 of all three taps are 24 consecutive elements of its channel's row
    typedef unsigned short u16x8 __attribute__((ext_vector_type(8)));
    auto sort_taps = [&](const unsigned char* src, bf16x8& t0, bf16x8& t1, bf16x8& t2, bool real) {
      u16x8 run[3];
#pragma unroll
      for (int i = 0; i < 3; ++i) run[i] = *reinterpret_cast<const u16x8*>(src + 16 * i);
      u16x8 w[3];
#pragma unroll
      for (int tap = 0; tap < 3; ++tap)
#pragma unroll
        for (int e = 0; e < 8; ++e) w[tap][e] = real ? run[(e * 3 + tap) / 8][(e * 3 + tap) % 8] : (unsigned short)0;
      t0 = __builtin_bit_cast(bf16x8, w[0]); t1 = __builtin_bit_cast(bf16x8, w[1]); t2 = __builtin_bit_cast(bf16x8, w[2]);
    };
    const unsigned char* img = lds + kBufB + hb * 48;
#pragma unroll
    for (int sl = 0; sl < 8; ++sl)
#pragma unroll
      for (int mb = 0; mb < 2; ++mb)
        sort_taps(img + (ql + 32 * mb) * ((kRawP1 + 1) * 16) + sl * 96, w1[0][sl][mb], w1[1][sl][mb], w1[2][sl][mb], true);
#pragma unroll
    for (int kk = 0; kk < 4; ++kk)
      sort_taps(img + kRawI1 * 1024 + ql * ((kRawP2 + 1) * 16) + kk * 96, w2[0][kk], w2[1][kk], w2[2][kk], true);
    // the third layer has 16 channels: the upper half of the MFMA rows is zero
#pragma unroll
    for (int kk = 0; kk < 2; ++kk)
      sort_taps(img + (kRawI1 + kRawI2) * 1024 + (ql & (C3 - 1)) * ((kRawP3 + 1) * 16) + kk * 96, w3[0][kk], w3[1][kk],
                w3[2][kk], ql < C3);
  } else {
    const unsigned char* wl = lds + kBufB + lane * 16;
#pragma unroll
    for (int tap = 0; tap < 3; ++tap)
#pragma unroll
      for (int sl = 0; sl < 8; ++sl)
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
          w1[tap][sl][mb] = *reinterpret_cast<const bf16x8*>(wl + ((tap * 8 + sl) * 2 + mb) * 1024);
#pragma unroll
    for (int tap = 0; tap < 3; ++tap)
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) w2[tap][kk] = *reinterpret_cast<const bf16x8*>(wl + (kBlocks1 + tap * 4 + kk) * 1024);
#pragma unroll
    for (int tap = 0; tap < 3; ++tap)
#pragma unroll
      for (int kk = 0; kk < 2; ++kk)
        w3[tap][kk] = *reinterpret_cast<const bf16x8*>(wl + (kBlocks1 + kBlocks2 + tap * 2 + kk) * 1024);
  }
  // pin them into their registers before the buffers they came through are refilled
#pragma unroll
  for (int tap = 0; tap < 3; ++tap) {
#pragma unroll
    for (int sl = 0; sl < 8; ++sl) asm volatile("" : "+v"(w1[tap][sl][0]), "+v"(w1[tap][sl][1]));
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) asm volatile("" : "+v"(w2[tap][kk]));
#pragma unroll
    for (int kk = 0; kk < 2; ++kk) asm volatile("" : "+v"(w3[tap][kk]));
  }
  __syncthreads();
  if (n_tiles > 1) issue_tile(1, 1);
  if (n_tiles > 2) issue_tile(2, 2);

  unsigned char* act_a = lds + kOffActA;
  unsigned char* act_b = lds + kOffActB;
  float* zmine = reinterpret_cast<float*>(lds + kOffZ) + row;
  f32x16 zero;
#pragma unroll
  for (int r = 0; r < 16; ++r) zero[r] = 0.f;

  // 1 for a position whose activations exist, 0 for one outside the sequence (or, in windows mode, on a padding row)
  auto inside_factor = [&](int pos) -> float {
    bool in = pos >= 0 && pos < n;
    if (a.row_valid != nullptr) {
      const int rel = in ? pos - base_row : 0;
      in = in && ((valid_bits[rel >> 5] >> (rel & 31)) & 1u);
    }
    return in ? 1.0f : 0.0f;
  };

  int buf = 0;
#pragma unroll 1
  for (int t = 0; t < n_tiles; ++t) {
    const int j0 = g0 + t * TMv;
    // tile t has landed once at most the loads of the tiles issued after it are still in flight (tiles t+1, t+2)
    if (t + 1 >= n_tiles) wait_loads();
    else if (t + 2 >= n_tiles) wait_loads_but<kLoadsPerWave>();
    else wait_loads_but<2 * kLoadsPerWave>();
    __syncthreads();       // tile t is in LDS; everyone is done with the previous tile's activations

    // ================= layer 1: 128 input channels (4 slices of keys, 4 of values), 64 output channels =============
    // the accumulators start from the bias: accumulator register 4*g4 + e of block mb is channel 32*mb + 8*g4 + 4*hb + e
    f32x16 acc0, acc1;
#pragma unroll
    for (int g4 = 0; g4 < 4; ++g4) {
      const f32x4 b0 = *reinterpret_cast<const f32x4*>(consts + 8 * g4 + 4 * hb);
      const f32x4 b1 = *reinterpret_cast<const f32x4*>(consts + 32 + 8 * g4 + 4 * hb);
#pragma unroll
      for (int e = 0; e < 4; ++e) { acc0[4 * g4 + e] = b0[e]; acc1[4 * g4 + e] = b1[e]; }
    }
    {
      const unsigned char* tb = lds + buf * kBufB;
#pragma unroll
      for (int tap = 0; tap < 3; ++tap) {
        // input row of this lane for the tap, and where its pieces sit: piece 2*(sl & 3) + hb of the key (sl < 4) or
        // value (sl >= 4) array is in slot (2*(sl & 3) + hb) ^ f, f = (r >> 1) & 7, i.e. at a0 ^ ((sl & 3) << 5)
        const int r = row + tap * a.d1;
        const int f = (r >> 1) & 7;
        const uint32_t a0 = (uint32_t)(r * kRowB + (((f >> 1) << 5) | ((hb ^ (f & 1)) << 4)));
        bf16x8 b[8];
#pragma unroll
        for (int sl = 0; sl < 8; ++sl)
          b[sl] = *reinterpret_cast<const bf16x8*>(tb + (a0 ^ (uint32_t)((sl & 3) << 5)) + (sl >= 4 ? kArrayB : 0));
#pragma unroll
        for (int sl = 0; sl < 8; ++sl) {
          acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(w1[tap][sl][0], b[sl], acc0, 0, 0, 0);
          acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(w1[tap][sl][1], b[sl], acc1, 0, 0, 0);
        }
      }
    }
    // Swish(acc), zero outside the sequence, as hi + lo bf16: the four channels of a group are half of 16-byte piece
    // 4*mb + g4 of this position's row.
    {
      const float inside = inside_factor(j0 - h1 + row);          // a factor, not a branch around the activation
      const int f = (row >> 1) & 7;
#pragma unroll
      for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4) {
          bf16x4 hi, lw;
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const float y = mb == 0 ? acc0[4 * g4 + e] : acc1[4 * g4 + e];
            const float val = silu_fast(y) * inside;
            hi[e] = static_cast<bf16_t>(val);
            lw[e] = static_cast<bf16_t>(val - static_cast<float>(hi[e]));
          }
          unsigned char* p = act_a + row * 128 + (((4 * mb + g4) ^ f) << 4) + 8 * hb;
          *reinterpret_cast<bf16x4*>(p) = hi;
          *reinterpret_cast<bf16x4*>(p + kPos * 128) = lw;
        }
    }
    __syncthreads();       // layer 1's output is complete; tile t's buffer is free
    if (t + 3 < n_tiles) issue_tile(t + 3, buf);
    buf = buf == kBufs - 1 ? 0 : buf + 1;

    // ================= layer 2: 64 -> 32 channels =====================================================================
#pragma unroll
    for (int g4 = 0; g4 < 4; ++g4) {
      const f32x4 b0 = *reinterpret_cast<const f32x4*>(consts + C1 + 8 * g4 + 4 * hb);
#pragma unroll
      for (int e = 0; e < 4; ++e) acc0[4 * g4 + e] = b0[e];
    }
#pragma unroll
    for (int tap = 0; tap < 3; ++tap) {
      int rr = row + tap * a.d2;               // input row of this position; rows past 127 belong to positions whose
      rr = rr < kPos ? rr : kPos - 1;          //   results are dropped: any finite data will do
      const int f = (rr >> 1) & 7;
      const unsigned char* p = act_a + rr * 128;
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        const uint32_t o = (uint32_t)(((2 * kk + hb) ^ f) << 4);
        const bf16x8 bh = *reinterpret_cast<const bf16x8*>(p + o);
        const bf16x8 bl = *reinterpret_cast<const bf16x8*>(p + o + kPos * 128);
        acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(w2[tap][kk], bh, acc0, 0, 0, 0);
        acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(w2[tap][kk], bl, acc0, 0, 0, 0);
      }
    }
    {
      const float inside = inside_factor(j0 - a.d3 + row);
      const int f = (row >> 2) & 3;            // 64-byte rows: four rows span the banks, so the swizzle steps every four
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {
        bf16x4 hi, lw;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float val = silu_fast(acc0[4 * g4 + e]) * inside;
          hi[e] = static_cast<bf16_t>(val);
          lw[e] = static_cast<bf16_t>(val - static_cast<float>(hi[e]));
        }
        unsigned char* p = act_b + row * 64 + ((g4 ^ f) << 4) + 8 * hb;
        *reinterpret_cast<bf16x4*>(p) = hi;
        *reinterpret_cast<bf16x4*>(p + kPos * 64) = lw;
      }
    }
    __syncthreads();       // layer 2's output is complete

    // ================= layer 3: 32 -> 16 channels (MFMA rows 16 .. 31 are zero weights), then the projection =======
    acc0 = zero;
#pragma unroll
    for (int g4 = 0; g4 < 2; ++g4) {           // channels 8*g4 + 4*hb + e < 16; the other rows' weights are zero
      const f32x4 b0 = *reinterpret_cast<const f32x4*>(consts + C1 + C2 + 8 * g4 + 4 * hb);
#pragma unroll
      for (int e = 0; e < 4; ++e) acc0[4 * g4 + e] = b0[e];
    }
#pragma unroll
    for (int tap = 0; tap < 3; ++tap) {
      int rr = row + tap * a.d3;
      rr = rr < kPos ? rr : kPos - 1;
      const int f = (rr >> 2) & 3;
      const unsigned char* p = act_b + rr * 64;
#pragma unroll
      for (int kk = 0; kk < 2; ++kk) {
        const uint32_t o = (uint32_t)(((2 * kk + hb) ^ f) << 4);
        const bf16x8 bh = *reinterpret_cast<const bf16x8*>(p + o);
        const bf16x8 bl = *reinterpret_cast<const bf16x8*>(p + o + kPos * 64);
        acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(w3[tap][kk], bh, acc0, 0, 0, 0);
        acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(w3[tap][kk], bl, acc0, 0, 0, 0);
      }
    }
    {
      float z = 0.f;
#pragma unroll
      for (int g4 = 0; g4 < 2; ++g4) {
        const f32x4 wo = *reinterpret_cast<const f32x4*>(consts + C1 + C2 + C3 + 8 * g4 + 4 * hb);
#pragma unroll
        for (int e = 0; e < 4; ++e) z = fmaf(silu_fast(acc0[4 * g4 + e]), wo[e], z);
      }
      z += __shfl_xor(z, 32, kWave);
      if (hb == 0) zmine[t * kPos] = z + bo;
    }
  }
  // every lane stores what it put there itself: no barrier
  for (int t = 0; t < n_tiles; ++t) {
    const int j = g0 + t * TMv + row;
    if (hb == 0 && row < TMv && j < n) a.logits[(int64_t)h * a.total + lo + j] = zmine[t * kPos];
  }
}

// panels[h][block][lane][e] = W_l[h][c][m][tap] with (l, tap, slice, channel block) from the block index as the kernel
// reads them, c = lane % 32 (+ 32 for the second channel block; 0 beyond c_out), m = 16*slice + 8*(lane / 32) + e
__global__ void __launch_bounds__(256)
score_deep_reg_panels_kernel(const uint16_t* __restrict__ W1, const uint16_t* __restrict__ W2,
                             const uint16_t* __restrict__ W3, uint16_t* __restrict__ panels, int64_t total) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= total) return;
  const int e = (int)(idx & 7), ln = (int)((idx >> 3) & 63);
  const int blk = (int)((idx >> 9) % kBlocks);
  const int64_t h = (idx >> 9) / kBlocks;
  const uint16_t* W;
  int cin, cout, tap, sl, c = ln & 31;
  if (blk < kBlocks1) { W = W1; cin = 2 * 64; cout = C1; tap = blk >> 4; sl = (blk >> 1) & 7; c += 32 * (blk & 1); }
  else if (blk < kBlocks1 + kBlocks2) { const int b = blk - kBlocks1; W = W2; cin = C1; cout = C2; tap = b >> 2; sl = b & 3; }
  else { const int b = blk - kBlocks1 - kBlocks2; W = W3; cin = C2; cout = C3; tap = b >> 1; sl = b & 1; }
  const int m = 16 * sl + 8 * (ln >> 5) + e;
  panels[idx] = c < cout ? W[((h * cout + c) * cin + m) * 3 + tap] : (uint16_t)0;
}

}  // namespace

// The paper's stack exactly: bf16, D = 64, three kernel-3 layers of 64, 32 and 16 channels; dilations such that a tile's
// input rows fit the buffers and at least half of a tile's positions are exact.
bool score_deep_reg_supported(const ltea_cfg& cfg, const ltea_cnn& cnn) {
  if (cfg.dtype != LTEA_BF16 || cfg.D != 64 || cnn.n_layers != 3) return false;
  for (int l = 0; l < 3; ++l)
    if (cnn.kernel[l] != 3 || cnn.dilation[l] < 1) return false;
  if (cnn.c_out[0] != C1 || cnn.c_out[1] != C2 || cnn.c_out[2] != C3) return false;
  static_assert(kMaxGroupTiles * kPos + 2 * kMaxD1 + 16 <= kScoreRowsPerDescriptor, "rows one workgroup addresses");
  return cnn.dilation[0] <= kMaxD1 && cnn.dilation[1] + cnn.dilation[2] <= 32;
}

hipError_t launch_score_deep_reg_panels(const ltea_cfg& cfg, const ltea_cnn& cnn, void* panels, hipStream_t stream) {
  const int64_t total = (int64_t)cfg.Hkv * kBlocks * 512;
  hipLaunchKernelGGL(score_deep_reg_panels_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream,
                     static_cast<const uint16_t*>(cnn.w[0]), static_cast<const uint16_t*>(cnn.w[1]),
                     static_cast<const uint16_t*>(cnn.w[2]), static_cast<uint16_t*>(panels), total);
  return hipGetLastError();
}

bool score_deep_reg_takes_raw_weights(const ltea_cnn& cnn) {
  return ((reinterpret_cast<uintptr_t>(cnn.w[0]) | reinterpret_cast<uintptr_t>(cnn.w[1]) |
           reinterpret_cast<uintptr_t>(cnn.w[2])) & 15u) == 0;
}

hipError_t launch_score_deep_reg(const ltea_cfg& cfg, const ltea_cnn& cnn, const void* k, const void* v, int64_t st,
                                 int64_t sh, const SeqView& sv, float* logits, const void* panels, hipStream_t stream,
                                 const uint8_t* row_valid) {
  if (sv.total_tokens == 0) return hipSuccess;
  DeepRegArgs a;
  a.k = static_cast<const bf16_t*>(k); a.v = static_cast<const bf16_t*>(v); a.st = st; a.sh = sh;
  a.panels = static_cast<const bf16_t*>(panels);    // null: the kernel sorts the caller's weight rows itself
  a.w1 = static_cast<const bf16_t*>(cnn.w[0]); a.w2 = static_cast<const bf16_t*>(cnn.w[1]);
  a.w3 = static_cast<const bf16_t*>(cnn.w[2]);
  if (panels == nullptr && !score_deep_reg_takes_raw_weights(cnn)) return hipErrorInvalidValue;
  a.bias1 = cnn.bias[0]; a.bias2 = cnn.bias[1]; a.bias3 = cnn.bias[2];
  a.w_out = static_cast<const bf16_t*>(cnn.w_out); a.b_out = cnn.b_out;
  a.d1 = cnn.dilation[0]; a.d2 = cnn.dilation[1]; a.d3 = cnn.dilation[2];
  a.cu = sv.cu_seqlens; a.n_seqs = sv.n_seqs; a.total = sv.total_tokens; a.logits = logits;
  a.row_valid = row_valid;
  const int TMv = kPos - 2 * (a.d2 + a.d3);
  a.group_tiles = pick_group_tiles(sv, cfg.Hkv, TMv, kMaxGroupTiles);
  a.Hkv = cfg.Hkv;
  const int64_t span = (int64_t)a.group_tiles * TMv;
  const int64_t groups_upper = (sv.total_tokens + span - 1) / span + sv.n_seqs;
  hipLaunchKernelGGL(score_deep_reg_kernel, dim3((unsigned)(groups_upper * cfg.Hkv)), dim3(kThreads), 0, stream, a);
  return hipGetLastError();
}

}  // namespace ltea
