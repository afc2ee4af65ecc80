// Prefill attention over window + retained set (paper Section 3.1.3) on bf16 MFMA for gfx950.
//
// Flash-attention-style tiling, two stages per query tile as in the paper's description: stage 1 walks
// 64-key tiles of the original K/V inside the tile's window range, stage 2 walks 64-slot tiles of the
// compact retained segment with a per-row mask "position <= i - window" (so entries still inside a
// query's window are never counted twice).  Per wave, tiles wholly outside its rows' reach are skipped and
// only tiles that straddle a window edge, the causal diagonal, the sequence end or the visibility frontier of
// the retained entries pay for masking.
//
// Work split: one workgroup = 128*QB consecutive queries of one (sequence, query head); 4 waves, each owning
// QB blocks of 32 queries (QB = 2 for D = 64, 1 for D = 128: what fits the register file at 2 waves/SIMD).
// MFMA shapes (v_mfma_f32_32x32x16_bf16, wave64):
//   S^T[key, query] = K[key, :] . Q[query, :]   A = K tile rows from LDS, B = Q fragment held in registers
//   O^T[d, query]  += V^T[d, key] . P^T[key, query]   A = V^T tile from LDS, B = P^T straight from S^T's
//                                                     accumulator registers (no shuffle, no LDS round trip)
// In the 32x32 accumulator layout a lane owns one query column, so the online-softmax statistics are
// per-lane scalars (the two lanes sharing a query exchange one value per 32 keys).  The contraction index of
// the second product is the key index; the rows of the K tile are fed to the first MFMA in a permuted
// order so that each lane's eight P values per MFMA are eight consecutive keys, which is what lets the
// V^T operand be read as one 16-byte LDS load.  V is transposed on its way into LDS (4 keys x 8 columns
// per thread, XOR-swizzled so that both the transposing stores and the operand loads spread over the 64 banks).
// K/V tiles are double-buffered in LDS and prefetched two tiles ahead through registers, one barrier per tile.
// The running maximum is only raised when a block of scores exceeds it by more than 2^8 (the result does not
// depend on the stabiliser), which keeps the accumulator rescale off the common path.
#include <type_traits>

#include "ltea_common.h"
#include "ltea_kernels.h"

namespace ltea {
namespace {

constexpr int BN = 64;   // keys per tile
constexpr int kThreads = 256;
constexpr float kLazyMax = 8.0f;  // log2 units

// Row of the K tile (within a block of 32) that MFMA row m must carry so that accumulator register r of
// lane half hb holds key 16*(r/8) + 8*hb + r%8: swap bits 2 and 3 of m.
__device__ __forceinline__ int key_row_of_mfma_row(int m) { return (m & 0x13) | ((m & 0x08) >> 1) | ((m & 0x04) << 1); }

// Both lane halves (l, l^32) receive max / sum of the pair.
__device__ __forceinline__ float pair_max(float x) {
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float pair_sum(float x) {
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
__device__ __forceinline__ int wave_min_i(int x) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) { const int y = __shfl_xor(x, off, kWave); x = y < x ? y : x; }
  return x;
}
__device__ __forceinline__ int wave_max_i(int x) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) { const int y = __shfl_xor(x, off, kWave); x = y > x ? y : x; }
  return x;
}

template <int D, int QB> struct Geo {
  static constexpr int BM = 128 * QB;           // queries per workgroup
  static constexpr int KS = D + 8;              // K tile row stride (elements); 16-byte pad
  static constexpr int VS = BN + 8;             // V^T tile row stride (elements)
  static constexpr int PPR = D / 8;             // 16-byte pieces per K row
  static constexpr int RPP = kThreads / PPR;    // K rows per pass
  static constexpr int KPASS = BN / RPP;        // passes over the K tile
  static constexpr int CPT = D / 16;            // V columns per thread (4 keys x CPT columns)
  static constexpr int OS = D + 8;              // epilogue staging row stride (elements)
  static constexpr int kBuf = BN * KS + D * VS; // elements per LDS tile buffer (K tile then V^T tile)
};

template <int D> struct TileRegs {
  u32x4 k[BN / (kThreads / (D / 8))];
  uint32_t v[4][D / 32];
  int pos;
};

template <int D, int QB>
__global__ void __launch_bounds__(kThreads, 2)
attention_mfma_kernel(const bf16_t* __restrict__ q, int64_t q_st, int64_t q_sh, const bf16_t* __restrict__ k,
                      const bf16_t* __restrict__ v, int64_t kv_st, int64_t kv_sh, const int32_t* __restrict__ cu,
                      int n_seqs, int tiles_upper, int n_work, int Hq, int Hkv, int window, int budget,
                      float scale_log2e, const bf16_t* __restrict__ k_ret, const bf16_t* __restrict__ v_ret,
                      const int32_t* __restrict__ ret_pos, const int32_t* __restrict__ ret_count,
                      bf16_t* __restrict__ out) {
  using G = Geo<D, QB>;
  using TR = TileRegs<D>;
  constexpr int BM = G::BM, KS = G::KS, VS = G::VS, kBuf = G::kBuf;
  static_assert(2 * kBuf >= BM * G::OS, "epilogue staging must fit in the tile buffers");
  __shared__ __align__(16) bf16_t lds[2 * kBuf];
  __shared__ int pos_lds[2][BN];
  __shared__ int pos_rng[2][2];   // min / max position of the tile's valid retained entries

  // ---- which (query head, sequence, query tile) is this workgroup? ------------------------------------
  // Workgroups are dealt round-robin to the 8 XCDs; give each XCD a contiguous range of work items so
  // that neighbouring query tiles of one head (which share most of their keys) meet in the same L2.
  const int per_xcd = (n_work + 7) / 8;
  const int work = (blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
  if (work >= n_work) return;
  const int hq = work / tiles_upper;
  int tile = work - hq * tiles_upper;
  int s = 0, n = 0;
  for (; s < n_seqs; ++s) {
    n = cu[s + 1] - cu[s];
    const int nt = (n + BM - 1) / BM;
    if (tile < nt) break;
    tile -= nt;
  }
  if (s == n_seqs) return;
  const int64_t lo = cu[s];
  const int h = hq / (Hq / Hkv);
  const int64_t head = (int64_t)s * Hkv + h;
  const int i0 = tile * BM;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int ql = lane & 31, hb = lane >> 5;
  const int r0 = i0 + 32 * QB * wv;         // first query row of this wave
  const int r_hi = r0 + 32 * QB - 1;        // last query row of this wave

  // ---- Q fragments (B operand of S^T): lane holds Q[row][16*ks + 8*hb .. +7] for its QB rows ------------
  bf16x8 qreg[QB][D / 16];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    const int qi = r0 + 32 * qb + ql;
    const int qc = qi < n ? qi : n - 1;
    const bf16_t* qrow = q + (lo + qc) * q_st + (int64_t)hq * q_sh;
#pragma unroll
    for (int ks = 0; ks < D / 16; ++ks) qreg[qb][ks] = *reinterpret_cast<const bf16x8*>(qrow + 16 * ks + 8 * hb);
  }

  // ---- tile schedule ------------------------------------------------------------------------------------
  const int i_last = (i0 + BM < n ? i0 + BM : n) - 1;            // last real query row of the workgroup
  const int jlo = i0 - window + 1 > 0 ? i0 - window + 1 : 0;
  const int jt0 = (jlo / BN) * BN;
  const int n_win_tiles = (i_last - jt0) / BN + 1;
  const int cnt = (budget > 0 && i_last - window >= 0) ? ret_count[head] : 0;
  const int n_ret_tiles = (cnt + BN - 1) / BN;
  const int n_tiles = n_win_tiles + n_ret_tiles;

  // ---- per-thread load addressing: buffer loads with 32-bit byte offsets; rows past the end of the sequence
  // (or past ret_count in the compact segment) are out of the descriptor's range and read as zeros ----------
  const uint32_t row_bytes = (uint32_t)kv_st * 2u;
  const uint32_t win_bytes = (uint32_t)(n - 1) * row_bytes + (uint32_t)(D * 2);
  const uint32_t ret_bytes = (uint32_t)cnt * (uint32_t)(D * 2);
  const auto rs_k = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t*>(k + lo * kv_st + (int64_t)h * kv_sh), 0, win_bytes, 0x00020000);
  const auto rs_v = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t*>(v + lo * kv_st + (int64_t)h * kv_sh), 0, win_bytes, 0x00020000);
  const auto rs_kr = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t*>(k_ret + head * budget * D), 0, ret_bytes, 0x00020000);
  const auto rs_vr = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t*>(v_ret + head * budget * D), 0, ret_bytes, 0x00020000);
  const int32_t* prbase = ret_pos + head * budget;
  const int k_piece = tid % G::PPR, k_row = tid / G::PPR;
  const int v_g = tid % 16, v_kg = tid / 16;   // 4 keys x CPT columns per thread; columns fastest across lanes
  const uint32_t k_col = (uint32_t)k_piece * 16u, v_col = (uint32_t)(v_g * G::CPT) * 2u;
  const uint32_t k_loc = (uint32_t)k_row * row_bytes + k_col;          // first pass; later passes add RPP rows
  const uint32_t v_loc = (uint32_t)(4 * v_kg) * row_bytes + v_col;     // key 4*v_kg; next keys add one row each
  const uint32_t kr_loc = (uint32_t)k_row * (uint32_t)(D * 2) + k_col;
  const uint32_t vr_loc = (uint32_t)(4 * v_kg) * (uint32_t)(D * 2) + v_col;

  auto load_rows = [&](const auto& rk, const auto& rv, uint32_t kb0, uint32_t vb0, uint32_t rb, TR& R) {
#pragma unroll
    for (int p = 0; p < G::KPASS; ++p)
      R.k[p] = __builtin_amdgcn_raw_buffer_load_b128(rk, kb0 + (uint32_t)(p * G::RPP) * rb, 0, 0);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      if constexpr (G::CPT == 8) {
        const u32x4 x = __builtin_amdgcn_raw_buffer_load_b128(rv, vb0 + (uint32_t)i * rb, 0, 0);
        R.v[i][0] = x[0]; R.v[i][1] = x[1]; R.v[i][2] = x[2]; R.v[i][3] = x[3];
      } else {
        const u32x2 x = __builtin_amdgcn_raw_buffer_load_b64(rv, vb0 + (uint32_t)i * rb, 0, 0);
        R.v[i][0] = x[0]; R.v[i][1] = x[1];
      }
    }
  };
  auto load_tile = [&](int t, TR& R) {
    if (t < n_win_tiles) {
      const uint32_t tb = (uint32_t)(jt0 + t * BN) * row_bytes;
      load_rows(rs_k, rs_v, tb + k_loc, tb + v_loc, row_bytes, R);
    } else {
      const int base = (t - n_win_tiles) * BN;
      const uint32_t tb = (uint32_t)base * (uint32_t)(D * 2);
      load_rows(rs_kr, rs_vr, tb + kr_loc, tb + vr_loc, (uint32_t)(D * 2), R);
      R.pos = 0x7FFFFFFF;
      if (tid < BN && base + tid < cnt) R.pos = prbase[base + tid];
    }
  };

  // LDS store addresses. V^T rows are d, columns keys; the 16-byte column chunk index is XOR-ed with
  // 2*((d >> 4) & 3) on both the store and the load side.
  const int v_d0 = v_g * G::CPT;
  const int k_st_off = k_row * KS + k_piece * 8;
  const int v_st_off = BN * KS + v_d0 * VS + ((4 * v_kg) ^ (16 * ((v_d0 >> 4) & 3)));
  auto store_tile = [&](int t, const TR& R) {
    bf16_t* buf = lds + (t & 1) * kBuf;
#pragma unroll
    for (int p = 0; p < G::KPASS; ++p) *reinterpret_cast<u32x4*>(buf + k_st_off + p * G::RPP * KS) = R.k[p];
#pragma unroll
    for (int c2 = 0; c2 < G::CPT / 2; ++c2) {
      const uint32_t a0 = R.v[0][c2], a1 = R.v[1][c2], a2 = R.v[2][c2], a3 = R.v[3][c2];
      u32x2 even, odd;
      even[0] = (a0 & 0xFFFFu) | (a1 << 16);
      even[1] = (a2 & 0xFFFFu) | (a3 << 16);
      odd[0] = (a0 >> 16) | (a1 & 0xFFFF0000u);
      odd[1] = (a2 >> 16) | (a3 & 0xFFFF0000u);
      *reinterpret_cast<u32x2*>(buf + v_st_off + (2 * c2) * VS) = even;
      *reinterpret_cast<u32x2*>(buf + v_st_off + (2 * c2 + 1) * VS) = odd;
    }
    if (t >= n_win_tiles && wv == 0) {   // wave 0 holds the tile's 64 positions (INT_MAX past ret_count)
      pos_lds[t & 1][lane] = R.pos;
      const int mn = wave_min_i(R.pos);
      const int mx = wave_max_i(R.pos == 0x7FFFFFFF ? (int)0x80000000 : R.pos);
      if (lane == 0) { pos_rng[t & 1][0] = mn; pos_rng[t & 1][1] = mx; }
    }
  };

  // operand load offsets inside a tile buffer
  const int a_k_off = key_row_of_mfma_row(ql) * KS + 8 * hb;                 // + 32*kb*KS + 16*ks
  const int s4 = ql >> 4;
  const int a_v_off0 = BN * KS + ql * VS + 8 * hb + 16 * (0 ^ s4);            // kk = 0
  const int a_v_off1 = BN * KS + ql * VS + 8 * hb + 16 * (1 ^ s4);            // kk = 1

  // ---- online softmax state (per lane = per query; the two lane halves keep separate partial sums) ------
  float m_run[QB], l_part[QB];
  f32x16 o[QB][D / 32];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    m_run[qb] = -INFINITY;
    l_part[qb] = 0.f;
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r) o[qb][db][r] = 0.f;
  }

  // mode: 0 = plain, 1 = window-edge mask (keys jt..), 2 = retained mask (positions in pos_lds).
  // The 64-key tile is consumed as two 32-key halves, each with its own softmax update, so that only one
  // 32x32 score block per query block is live at a time.
  auto compute = [&](const int mode, const bf16_t* buf, const int* pos, int jt) {
    const bf16_t* a_k = buf + a_k_off;
    const bf16_t* a_v0 = buf + a_v_off0;
    const bf16_t* a_v1 = buf + a_v_off1;
    // Both 32-key score blocks are issued before the first one is consumed, so the matrix pipe keeps working on
    // the second block (and later on the first block's P.V product) while the VALU runs the softmax.
    f32x16 sacc[2][QB];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
      for (int qb = 0; qb < QB; ++qb)
#pragma unroll
        for (int r = 0; r < 16; ++r) sacc[kb][qb][r] = 0.f;
#pragma unroll
      for (int ks = 0; ks < D / 16; ++ks) {
        const bf16x8 a = *reinterpret_cast<const bf16x8*>(a_k + 32 * kb * KS + 16 * ks);
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
          sacc[kb][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qreg[qb][ks], sacc[kb][qb], 0, 0, 0);
      }
    }
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
      bf16x8 pb[QB][2];
#pragma unroll
      for (int qb = 0; qb < QB; ++qb) {
        f32x16& sc = sacc[kb][qb];
        const int qi = r0 + 32 * qb + ql;
        // register r is key (local) 32*kb + 16*(r/8) + 8*hb + r%8
        if (mode == 1) {
          // valid local keys c (without the 8*hb term) form the range [c_lo, c_hi]: causal, window and sequence end
          const int shift = jt + 8 * hb;
          int c_hi = qi - shift;                                   // j <= qi
          const int c_end = n - 1 - shift;                         // j <= n-1
          c_hi = c_hi < c_end ? c_hi : c_end;
          int c_lo = qi - window + 1 - shift;                      // j >= qi - window + 1
          const unsigned span = c_hi >= c_lo ? (unsigned)(c_hi - c_lo) : 0u;
          if (c_hi < c_lo) c_lo = 0x40000000;                      // nothing valid
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int c = 32 * kb + 16 * (r / 8) + (r % 8);
            sc[r] = ((unsigned)(c - c_lo) <= span) ? sc[r] : -INFINITY;
          }
        } else if (mode == 2) {
          const int lim = qi - window;
#pragma unroll
          for (int r8 = 0; r8 < 2; ++r8) {
            const int* pp = pos + 32 * kb + 16 * r8 + 8 * hb;
#pragma unroll
            for (int e = 0; e < 8; ++e) sc[8 * r8 + e] = (pp[e] <= lim) ? sc[8 * r8 + e] : -INFINITY;
          }
        }
        // ---- online softmax with a lazily raised maximum ----------------------------------------------------
        float mx = fmaxf(sc[0], sc[1]);
#pragma unroll
        for (int r = 2; r < 16; r += 2) mx = fmaxf(fmaxf(mx, sc[r]), sc[r + 1]);
        mx = pair_max(mx);
        const float mcand = mx * scale_log2e;
        const bool grow = mcand > m_run[qb] + kLazyMax;   // true on the first visible keys (m_run = -inf)
        if (__builtin_amdgcn_ballot_w64(grow) != 0ull) {
          const float alpha = grow ? __builtin_amdgcn_exp2f(m_run[qb] - mcand) : 1.0f;
          m_run[qb] = grow ? mcand : m_run[qb];
          l_part[qb] *= alpha;
#pragma unroll
          for (int db = 0; db < D / 32; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) o[qb][db][r] *= alpha;
        }
        const float m_use = (m_run[qb] == -INFINITY) ? 0.f : m_run[qb];
        float psum0 = 0.f, psum1 = 0.f;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const float p = __builtin_amdgcn_exp2f(fmaf(sc[r], scale_log2e, -m_use));
          if (r & 1) psum1 += p; else psum0 += p;
          pb[qb][r / 8][r % 8] = static_cast<bf16_t>(p);
        }
        l_part[qb] += psum0 + psum1;
      }
      // ---- O^T += V^T P^T -----------------------------------------------------------------------------------
#pragma unroll
      for (int db = 0; db < D / 32; ++db) {
        const int col = 32 * (kb ^ (db & 1));
        const bf16x8 a0 = *reinterpret_cast<const bf16x8*>(a_v0 + 32 * db * VS + col);
        const bf16x8 a1 = *reinterpret_cast<const bf16x8*>(a_v1 + 32 * db * VS + col);
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
          o[qb][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, pb[qb][0], o[qb][db], 0, 0, 0);
          o[qb][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, pb[qb][1], o[qb][db], 0, 0, 0);
        }
      }
    }
  };

  // ---- software pipeline: tile t is computed from LDS buffer t&1 while tile t+1 is being stored into the other
  // buffer and tile t+2 is in flight from global memory --------------------------------------------------------
  TR regs;
  load_tile(0, regs);
  store_tile(0, regs);
  if (n_tiles > 1) load_tile(1, regs);
  for (int t = 0; t < n_tiles; ++t) {
    __syncthreads();   // tile t is in LDS; everyone is done with tile t-1 (whose buffer is overwritten next)
    if (t + 1 < n_tiles) store_tile(t + 1, regs);
    if (t + 2 < n_tiles) load_tile(t + 2, regs);
    const bf16_t* buf = lds + (t & 1) * kBuf;
    // classify the tile for this wave: -1 skip, 0 every (query, key) pair valid, 1 window-edge mask, 2 retained mask
    int mode = -1, jt = 0;
    if (r0 < n) {
      if (t < n_win_tiles) {
        jt = jt0 + t * BN;
        // keys this wave can use at all: [r0 - window + 1, r_hi]
        if (!(jt > r_hi || jt + BN - 1 < r0 - window + 1))
          mode = ((jt + BN - 1 <= r0) && (jt >= r_hi - window + 1)) ? 0 : 1;
      } else {
        const int pmin = pos_rng[t & 1][0], pmax = pos_rng[t & 1][1];
        if (pmin <= r_hi - window) {                     // some entry has left one of this wave's windows
          const bool full = (t - n_win_tiles + 1) * BN <= cnt;
          mode = (full && pmax <= r0 - window) ? 0 : 2;
        }
      }
    }
    mode = __builtin_amdgcn_readfirstlane(mode);
    if (mode >= 0) compute(mode, buf, pos_lds[t & 1], jt);
  }

  // ---- epilogue: normalise, stage through LDS, store rows coalesced -------------------------------------------
  __syncthreads();  // tile buffers are free
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    const float inv = 1.0f / pair_sum(l_part[qb]);
    bf16_t* orow = lds + (32 * QB * wv + 32 * qb + ql) * G::OS + 4 * hb;
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {
        bf16x4 w4;
#pragma unroll
        for (int e = 0; e < 4; ++e) w4[e] = static_cast<bf16_t>(o[qb][db][4 * g4 + e] * inv);
        *reinterpret_cast<bf16x4*>(orow + 32 * db + 8 * g4) = w4;
      }
  }
  __syncthreads();
  {
    bf16_t* obase = out + ((lo + i0) * Hq + hq) * D;
    const int64_t orow_stride = (int64_t)Hq * D;
#pragma unroll
    for (int p = 0; p < BM / G::RPP; ++p) {
      const int row = p * G::RPP + k_row;
      if (i0 + row < n)
        *reinterpret_cast<u32x4*>(obase + row * orow_stride + k_piece * 8) =
            *reinterpret_cast<const u32x4*>(lds + row * G::OS + k_piece * 8);
    }
  }
}

template <int D, int QB>
hipError_t run(const ltea_cfg& cfg, const void* q, int64_t q_st, int64_t q_sh, const void* k, const void* v,
               int64_t kv_st, int64_t kv_sh, const SeqView& sv, const ltea_cache& c, void* out, hipStream_t stream) {
  constexpr int BM = Geo<D, QB>::BM;
  const float scale = cfg.softmax_scale > 0.f ? cfg.softmax_scale : 1.0f / sqrtf((float)cfg.D);
  const int64_t tiles_upper = (sv.total_tokens + BM - 1) / BM + sv.n_seqs;
  const int64_t n_work = tiles_upper * cfg.Hq;
  const int64_t grid = (n_work + 7) / 8 * 8;
  hipLaunchKernelGGL((attention_mfma_kernel<D, QB>), dim3((unsigned)grid), dim3(kThreads), 0, stream,
                     static_cast<const bf16_t*>(q), q_st, q_sh, static_cast<const bf16_t*>(k),
                     static_cast<const bf16_t*>(v), kv_st, kv_sh, sv.cu_seqlens, sv.n_seqs, (int)tiles_upper,
                     (int)n_work, cfg.Hq, cfg.Hkv, cfg.window, cfg.budget, scale * 1.4426950408889634f,
                     static_cast<const bf16_t*>(c.k_ret), static_cast<const bf16_t*>(c.v_ret), c.ret_pos, c.ret_count,
                     static_cast<bf16_t*>(out));
  return hipGetLastError();
}

}  // namespace

// The kernel addresses K/V rows of one sequence with 32-bit byte offsets.
bool attention_mfma_supported(const ltea_cfg& cfg, int64_t kv_stride_tok, int32_t max_seqlen) {
  if (cfg.dtype != LTEA_BF16 || (cfg.D != 64 && cfg.D != 128)) return false;
  return (int64_t)max_seqlen * kv_stride_tok * 2 < ((int64_t)1 << 31) && (int64_t)cfg.budget * cfg.D * 2 < ((int64_t)1 << 31);
}

hipError_t launch_attention_mfma(const ltea_cfg& cfg, const void* q, int64_t q_st, int64_t q_sh, const void* k,
                                 const void* v, int64_t kv_st, int64_t kv_sh, const SeqView& sv, const ltea_cache& c,
                                 void* out, hipStream_t stream) {
  if (sv.total_tokens == 0) return hipSuccess;
  return cfg.D == 64 ? run<64, 1>(cfg, q, q_st, q_sh, k, v, kv_st, kv_sh, sv, c, out, stream)
                     : run<128, 1>(cfg, q, q_st, q_sh, k, v, kv_st, kv_sh, sv, c, out, stream);
}

}  // namespace ltea
