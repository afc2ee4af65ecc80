// Prefill attention over window + retained set (paper Section 3.1.3) on bf16 MFMA for gfx950.
//
// Flash-attention-style tiling, two stages per query tile as in the paper's description: stage 1 walks
// 64-key tiles of the original K/V inside the tile's window range, stage 2 walks 64-slot tiles of the
// compact retained segment with a per-row mask "position <= i - window" (so entries still inside a
// query's window are never counted twice).  Per wave, tiles wholly outside its rows' reach are skipped and
// only tiles that straddle a window edge, the causal diagonal, the sequence end or the visibility frontier of
// the retained entries pay for masking.
//
// Work split: one workgroup = 128 consecutive queries of one (sequence, query head), 4 waves each owning a block
// of 32 queries; or, for grouped-query shapes, the same 32 queries of four query heads that share a KV head, one
// head per wave.  MFMA shapes (v_mfma_f32_32x32x16_bf16, wave64):
//   S^T[key, query] = K[key, :] . Q[query, :]   A = K tile rows from LDS, B = Q fragment held in registers
//   O^T[d, query]  += V^T[d, key] . P^T[key, query]   A = V^T fragments from LDS, B = P^T straight from S^T's
//                                                     accumulator registers (no shuffle, no LDS round trip)
// In the 32x32 accumulator layout a lane owns one query column, so the softmax statistics are per-lane scalars
// (the two lanes sharing a query keep separate partial sums and meet once, in the epilogue).  The contraction index of
// the second product is the key index; the rows of the K tile are fed to the first MFMA in a permuted
// order so that each lane's eight P values per MFMA are eight consecutive keys.  V stays row-major in LDS
// and its A operand (eight consecutive keys of one column per lane) comes out of the transposing LDS load
// ds_read_b64_tr_b16, two per MFMA; the tile's 64-byte chunks are XOR-swizzled so that those loads and the
// staging stores spread over the 64 banks without padding.
// K/V tiles are double-buffered in LDS and prefetched one tile ahead through registers, one barrier per tile
// (three workgroups share a CU at D = 64, two at D = 128; a 128-VGPR build of the D = 64 kernel reaches four but
// spills, which costs HBM traffic and gains no time).  There is no running maximum: a row's exponentials are taken
// relative to the maximum of the first block in which it sees a key (the result does not depend on that reference
// value as long as the exponentials stay in range; a workgroup whose row sums leave the range repeats its tiles with
// the exact running maximum), which keeps the row-maximum reduction and the accumulator rescale off the common path.
// Inside a tile the matrix work of one 32-key block is placed next to the
// exponentials of the other, so that they overlap within the wave's in-order instruction stream.
#include <type_traits>

#include "ltea_common.h"
#include "ltea_kernels.h"
#include "mfma_tiles.h"

namespace ltea {
namespace {

constexpr int BN = 64;   // keys per tile
constexpr int kThreads = 256;
constexpr float kBig = 1.8446744e19f;  // 2^64: a row sum above this (or not a number) sends the workgroup through its tiles again

template <int D, int QB> struct Geo {
  static constexpr int BM = 128 * QB;           // queries per workgroup
  static constexpr int KS = D + 8;              // K tile row stride (elements); 16-byte pad
  static constexpr int VS = D;                  // V tile row stride (elements): unpadded, 64-byte chunks swizzled
  static constexpr int PPR = D / 8;             // 16-byte pieces per K row
  static constexpr int RPP = kThreads / PPR;    // K rows per pass
  static constexpr int KPASS = BN / RPP;        // passes over the K tile
  static constexpr int OS = D + 8;              // epilogue staging row stride (elements)
  static constexpr int kBuf = BN * KS + BN * VS; // elements per LDS tile buffer (K tile then V tile)
};

template <int D> struct TileRegs {
  u32x4 k[BN / (kThreads / (D / 8))];
  u32x4 v[BN / (kThreads / (D / 8))];
  int pos;
};

// HW = query heads per workgroup.  1: the four waves take four consecutive blocks of 32 query positions of one head.
// 4 (grouped-query shapes with a multiple of four query heads per KV head): the four waves take the SAME 32 positions
// of four query heads that share the KV head.  The K/V tiles are shared either way, but with HW = 4 every wave sees the
// same window, so a tile is plain, masked or out of reach for all four at once (with HW = 1 the waves' windows are
// shifted by 32 positions each, the workgroup's key range is 96 positions longer, and whenever one wave has a masked
// tile the other three wait for it at the tile barrier).
template <int D, int QB, int HW>
__global__ void __launch_bounds__(kThreads, D == 64 ? 3 : 2)
attention_mfma_kernel(const bf16_t* __restrict__ q, int64_t q_st, int64_t q_sh, const bf16_t* __restrict__ k,
                      const bf16_t* __restrict__ v, int64_t kv_st, int64_t kv_sh, const int32_t* __restrict__ cu,
                      int n_seqs, int tiles_upper, int n_work, int Hq, int Hkv, int window, int budget,
                      float scale_log2e, const bf16_t* __restrict__ k_ret, const bf16_t* __restrict__ v_ret,
                      const int32_t* __restrict__ ret_pos, const int32_t* __restrict__ ret_count,
                      bf16_t* __restrict__ out, const int32_t* __restrict__ kv_start,
                      const int32_t* __restrict__ kv_len, float* __restrict__ lse, int64_t lse_stride) {
  using G = Geo<D, QB>;
  using TR = TileRegs<D>;
  constexpr int BM = G::BM, KS = G::KS, VS = G::VS, kBuf = G::kBuf;
  constexpr int BMQ = BM / HW;     // query positions per workgroup (BM = rows of all its waves)
  static_assert(HW == 1 || HW == 4, "one head, or one head per wave");
  static_assert(2 * kBuf >= BM * G::OS, "epilogue staging must fit in the tile buffers");
  __shared__ __align__(16) bf16_t lds[2 * kBuf];
  __shared__ int pos_lds[2][BN];
  __shared__ int redo_flag;

  // ---- which (query head, sequence, query tile) is this workgroup? ------------------------------------
  // Workgroups are dealt round-robin to the 8 XCDs; give each XCD a contiguous range of work items so
  // that neighbouring query tiles of one head (which share most of their keys) meet in the same L2.  When the heads
  // divide evenly over the XCDs, an XCD takes whole heads and walks them tile by tile, heads fastest, long tiles first:
  // the first tiles of every sequence, whose window is still filling, come last and fill the gaps when the grid drains.
  const int per_xcd = (n_work + 7) / 8;
  const int work = (blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
  if (work >= n_work) return;
  int unit, flat_tile;                      // unit = query head (HW = 1) or group of HW query heads
  const int units = Hq / HW;
  const bool whole_heads = units % 8 == 0;
  if (whole_heads) {
    const int hpx = units / 8, in_xcd = blockIdx.x / 8;      // per_xcd == hpx * tiles_upper
    unit = (blockIdx.x % 8) * hpx + in_xcd % hpx;
    flat_tile = in_xcd / hpx;
  } else {
    unit = work / tiles_upper;
    flat_tile = work - unit * tiles_upper;
  }
  // cu packs the query / output rows.  Normally it packs the keys as well; with kv_start / kv_len given, the keys
  // of sequence s are rows kv_start[s] .. kv_start[s] + kv_len[s] - 1 of k / v and the queries are the last
  // cu[s+1] - cu[s] positions of that key sequence (continuation of a prefill).
  int tile, s, n, lo_q;
  if (whole_heads && kv_start == nullptr) {
    if (!locate_tile_late_first(cu, n_seqs, BMQ, (window + BMQ - 1) / BMQ, flat_tile, s, tile, lo_q, n)) return;
  } else {
    if (!locate_tile(cu, n_seqs, BMQ, flat_tile, s, tile, lo_q, n)) return;
  }
  int64_t lo = lo_q;
  int q_begin = 0;
  if (kv_start != nullptr) {
    const int nq = n;
    lo = kv_start[s];
    n = kv_len[s];
    q_begin = n - nq;
  }
  const int h = (unit * HW) / (Hq / Hkv);
  const int64_t head = (int64_t)s * Hkv + h;
  const int i0 = q_begin + tile * BMQ;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int ql = lane & 31, hb = lane >> 5;
  const int hq = HW == 1 ? unit : unit * HW + wv;                 // this wave's query head
  const int r0 = i0 + (HW == 1 ? 32 * QB * wv : 0);               // first query row of this wave
  const int r_hi = r0 + 32 * QB - 1;        // last query row of this wave

  // ---- Q fragments (B operand of S^T): lane holds Q[row][16*ks + 8*hb .. +7] for its QB rows ------------
  bf16x8 qreg[QB][D / 16];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    const int qi = r0 + 32 * qb + ql;
    const int qc = qi < n ? qi : n - 1;
    const bf16_t* qrow = q + (int64_t)(lo_q + qc - q_begin) * q_st + (int64_t)hq * q_sh;
#pragma unroll
    for (int ks = 0; ks < D / 16; ++ks) qreg[qb][ks] = *reinterpret_cast<const bf16x8*>(qrow + 16 * ks + 8 * hb);
  }

  // ---- tile schedule ------------------------------------------------------------------------------------
  const int i_last = (i0 + BMQ < n ? i0 + BMQ : n) - 1;          // last real query row of the workgroup
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
  const uint32_t k_col = (uint32_t)k_piece * 16u;
  const uint32_t k_loc = (uint32_t)k_row * row_bytes + k_col;          // first pass; later passes add RPP rows
  const uint32_t kr_loc = (uint32_t)k_row * (uint32_t)(D * 2) + k_col;

  auto load_rows = [&](const auto& rk, const auto& rv, uint32_t b0, uint32_t rb, TR& R) {
#pragma unroll
    for (int p = 0; p < G::KPASS; ++p) {
      R.k[p] = __builtin_amdgcn_raw_buffer_load_b128(rk, b0 + (uint32_t)(p * G::RPP) * rb, 0, 0);
      R.v[p] = __builtin_amdgcn_raw_buffer_load_b128(rv, b0 + (uint32_t)(p * G::RPP) * rb, 0, 0);
    }
  };
  auto load_tile = [&](int t, TR& R) {
    if (t < n_win_tiles) {
      const uint32_t tb = (uint32_t)(jt0 + t * BN) * row_bytes;
      load_rows(rs_k, rs_v, tb + k_loc, row_bytes, R);
    } else {
      const int base = (t - n_win_tiles) * BN;
      const uint32_t tb = (uint32_t)base * (uint32_t)(D * 2);
      load_rows(rs_kr, rs_vr, tb + kr_loc, (uint32_t)(D * 2), R);
      R.pos = 0x7FFFFFFF;
      if (tid < BN && base + tid < cnt) R.pos = prbase[base + tid];
    }
  };

  // LDS store addresses. The V tile stays row-major [key][d] without padding; its 64-byte chunks (32 columns)
  // are XOR-swizzled with the key row so that the transposing operand loads (4 keys x 16 columns per 16 lanes)
  // spread over all banks.  Rows of one pass differ by multiples of RPP, which leaves the swizzle term unchanged.
  static_assert(G::RPP % 4 == 0, "row passes must preserve the swizzle phase");
  const int k_st_off = k_row * KS + k_piece * 8;
  const int v_st_off = BN * KS + k_row * VS + (((k_piece >> 2) ^ chunk_swizzle<D>(k_row)) << 5) + (k_piece & 3) * 8;
  auto store_tile = [&](int t, const TR& R) {
    bf16_t* buf = lds + (t & 1) * kBuf;
#pragma unroll
    for (int p = 0; p < G::KPASS; ++p) {
      *reinterpret_cast<u32x4*>(buf + k_st_off + p * G::RPP * KS) = R.k[p];
      *reinterpret_cast<u32x4*>(buf + v_st_off + p * G::RPP * VS) = R.v[p];
    }
    if (t >= n_win_tiles && wv == 0) pos_lds[t & 1][lane] = R.pos;   // the tile's 64 positions (INT_MAX past ret_count)
  };

  // operand load offsets inside a tile buffer
  const int a_k_off = tile_row_of_mfma_row(ql) * KS + 8 * hb;                 // + 32*kb*KS + 16*ks
  // V operand through the transposing LDS load: in each group of 16 lanes, lane j points at the four columns
  // d0 + 4*(j%4).. of key row kbase + j/4, and receives column d0 + j of the four keys kbase..kbase+3.
  const int tr_key = 8 * hb + ((lane & 15) >> 2);           // + 32*kb + 16*kk (+ 4 for the upper half)
  const int tr_col = 16 * ((lane >> 4) & 1) + 4 * (lane & 3);  // + 32*db, inside one 64-byte chunk
  const int tr_swz = chunk_swizzle<D>(tr_key);                  // unchanged by adding multiples of 4 to the key
  const int a_v_off = BN * KS + tr_key * VS + tr_col;

  // ---- softmax state (per lane = per query; the two lane halves keep separate partial sums) ------
  float m_run[QB], l_part[QB];
  bool all_have_m = false;     // wave-uniform: every row of the wave has a reference value (m_run finite)
  bool exact_pass = false;     // workgroup-uniform: second run over the tiles, with the running maximum in every block
  f32x16 o[QB][D / 32];
  auto reset_rows = [&]() {
    all_have_m = false;
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
      m_run[qb] = -INFINITY;
      l_part[qb] = 0.f;
#pragma unroll
      for (int db = 0; db < D / 32; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[qb][db][r] = 0.f;
    }
  };
  reset_rows();

  // mode: 0 = plain, 1 = window-edge mask (keys jt..), 2 = retained mask (positions in pos_lds).
  // The 64-key tile is consumed as two 32-key halves, each with its own softmax update, so that only one
  // 32x32 score block per query block is live at a time.
  auto compute = [&](const int mode, const bf16_t* buf, const int* pos, int jt) {
    const bf16_t* a_k = buf + a_k_off;
    const bf16_t* a_v = buf + a_v_off;
    // The tile is consumed as two 32-key blocks.  Program order puts the matrix work of one block next to the
    // exponentials of the other (scores of block 1 beside the softmax of block 0, P.V of block 0 beside the
    // softmax of block 1), because a wave issues in order: only MFMAs that sit between VALU instructions in
    // the instruction stream run concurrently with them.
    auto load_k_ops = [&](int kb, bf16x8 (&a)[D / 16]) {
#pragma unroll
      for (int ks = 0; ks < D / 16; ++ks) a[ks] = *reinterpret_cast<const bf16x8*>(a_k + 32 * kb * KS + 16 * ks);
    };
    auto score_block = [&](const bf16x8 (&a)[D / 16], f32x16 (&sc)[QB]) {
#pragma unroll
      for (int qb = 0; qb < QB; ++qb)
#pragma unroll
        for (int r = 0; r < 16; ++r) sc[qb][r] = 0.f;
#pragma unroll
      for (int ks = 0; ks < D / 16; ++ks)
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
          sc[qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[ks], qreg[qb][ks], sc[qb], 0, 0, 0);
    };
    // mask: register r is local key 32*kb + 16*(r/8) + 8*hb + r%8
    auto apply_mask = [&](int kb, f32x16 (&scs)[QB]) {
#pragma unroll
      for (int qb = 0; qb < QB; ++qb) {
        f32x16& sc = scs[qb];
        const int qi = r0 + 32 * qb + ql;
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
      }
    };
    // The reference value m of a row (probabilities are exp2(score - m)) only has to keep the exponentials in range,
    // so it is not the running maximum: a row takes the maximum of the first block in which it sees a key and keeps it
    // (l is then at least the 1 of that block, and the softmax is the same function of the scores for any m).  Scores
    // that later exceed m by more than the exponent range allows show up as a huge or non-finite row sum when the
    // tiles are done; the workgroup then runs its tiles a second time with the exact running maximum in every block.
    auto raise_reference = [&](const f32x16 (&scs)[QB]) {
      bool still_none = false;
#pragma unroll
      for (int qb = 0; qb < QB; ++qb) {
        const f32x16& sc = scs[qb];
        float mx = fmaxf(sc[0], sc[1]);
#pragma unroll
        for (int r = 2; r < 16; r += 2) mx = fmaxf(fmaxf(mx, sc[r]), sc[r + 1]);
        mx = pair_max(mx);
        const float m_new = fmaxf(m_run[qb], mx * scale_log2e);
        // nothing visible so far and nothing now: m stays -inf, and the factor must not become exp2(nan)
        const float a = (m_new == m_run[qb]) ? 1.0f : __builtin_amdgcn_exp2f(m_run[qb] - m_new);
        m_run[qb] = m_new;
        l_part[qb] *= a;
        if (__builtin_amdgcn_ballot_w64(a != 1.0f) != 0ull) {
#pragma unroll
          for (int db = 0; db < D / 32; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) o[qb][db][r] *= a;
        }
        still_none = still_none || (m_new == -INFINITY);
      }
      all_have_m = __builtin_amdgcn_ballot_w64(still_none) == 0ull;
    };
    auto exp_block = [&](const f32x16 (&scs)[QB], bf16x8 (&pb)[QB][2], float (&psum)[QB]) {
#pragma unroll
      for (int qb = 0; qb < QB; ++qb) {
        const float m_use = (m_run[qb] == -INFINITY) ? 0.f : m_run[qb];
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const float p = __builtin_amdgcn_exp2f(fmaf(scs[qb][r], scale_log2e, -m_use));
          pb[qb][r / 8][r % 8] = static_cast<bf16_t>(p);
        }
        // Row sum from the rounded probabilities, two per instruction (v_dot2c_f32_bf16 with a vector of ones):
        // the denominator then matches the bf16 P that the second MFMA consumes.
        bf16x2 ones;
        ones[0] = static_cast<bf16_t>(1.0f); ones[1] = static_cast<bf16_t>(1.0f);
        float psum0 = 0.f, psum1 = 0.f;
#pragma unroll
        for (int r2 = 0; r2 < 8; r2 += 2) {
          bf16x2 e0, e1;
          e0[0] = pb[qb][r2 / 4][(2 * r2) % 8]; e0[1] = pb[qb][r2 / 4][(2 * r2) % 8 + 1];
          e1[0] = pb[qb][r2 / 4][(2 * r2) % 8 + 2]; e1[1] = pb[qb][r2 / 4][(2 * r2) % 8 + 3];
          psum0 = __builtin_amdgcn_fdot2_f32_bf16(e0, ones, psum0, false);
          psum1 = __builtin_amdgcn_fdot2_f32_bf16(e1, ones, psum1, false);
        }
        psum[qb] = psum0 + psum1;
      }
    };
    // Softmax of one 32-key block whose (masked) scores are in s: probabilities to p, row sums to l_part
    auto softmax_block = [&](int kb, f32x16 (&s)[QB], bf16x8 (&p)[QB][2]) {
      float psum[QB];
      if (!all_have_m || exact_pass) raise_reference(s);
      exp_block(s, p, psum);
#pragma unroll
      for (int qb = 0; qb < QB; ++qb) {
        l_part[qb] += psum[qb];
        // Pin the packed probabilities here: without a use in this block the compiler sinks the exponentials
        // past the following branches, away from the MFMAs they are meant to overlap with.
        u32x4 w0 = __builtin_bit_cast(u32x4, p[qb][0]), w1 = __builtin_bit_cast(u32x4, p[qb][1]);
        asm volatile("" : "+v"(w0), "+v"(w1), "+v"(l_part[qb]));
        p[qb][0] = __builtin_bit_cast(bf16x8, w0);
        p[qb][1] = __builtin_bit_cast(bf16x8, w1);
      }
    };
    auto load_v_ops = [&](int kb, bf16x8 (&av)[D / 32][2]) {
#pragma unroll
      for (int db = 0; db < D / 32; ++db) {
        const bf16_t* ap = a_v + 32 * kb * VS + ((db ^ tr_swz) << 5);
        av[db][0] = load_transposed(ap, VS);
        av[db][1] = load_transposed(ap + 16 * VS, VS);
      }
    };
    auto pv_block = [&](const bf16x8 (&av)[D / 32][2], const bf16x8 (&pb)[QB][2]) {   // O^T += V^T P^T
#pragma unroll
      for (int db = 0; db < D / 32; ++db)
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
          o[qb][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[db][0], pb[qb][0], o[qb][db], 0, 0, 0);
          o[qb][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[db][1], pb[qb][1], o[qb][db], 0, 0, 0);
        }
    };
    // The value operands are requested ahead of the exponentials that hide their LDS latency (measured against
    // requesting them next to their MFMAs: 2 % at D = 128, 1 % at D = 64).
    constexpr bool kEarlyV = true;
    f32x16 s0[QB], s1[QB];
    bf16x8 p0[QB][2], p1[QB][2];
    bf16x8 ak0[D / 16], ak1[D / 16];
    load_k_ops(0, ak0);
    load_k_ops(1, ak1);        // requested together with block 0's operands: their LDS latency passes under block 0
    __builtin_amdgcn_sched_group_barrier(0x100, 2 * (D / 16), 0);   // all operand reads first
    score_block(ak0, s0);
    apply_mask(0, s0);
    score_block(ak1, s1);
    bf16x8 av0[D / 32][2], av1[D / 32][2];
    if constexpr (kEarlyV) load_v_ops(0, av0);
    softmax_block(0, s0, p0);
    apply_mask(1, s1);
    if constexpr (kEarlyV) load_v_ops(1, av1);
    else load_v_ops(0, av0);
    pv_block(av0, p0);
    softmax_block(1, s1, p1);   // if it scales the accumulators, block 0's product (formed under the old m) is in them
    if constexpr (!kEarlyV) load_v_ops(1, av1);
    pv_block(av1, p1);
  };

  // ---- software pipeline: tile t is computed from LDS buffer t&1 while tile t+1 is being stored into the other
  // buffer and tile t+2 is in flight from global memory --------------------------------------------------------
  auto step = [&](int t, TR& R) {   // R holds tile t+1 on entry and tile t+2 on exit
    __syncthreads();   // tile t is in LDS; everyone is done with tile t-1 (whose buffer is overwritten next)
    if (t + 1 < n_tiles) store_tile(t + 1, R);
    if (t + 2 < n_tiles) load_tile(t + 2, R);
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
        // every wave looks at the tile's positions itself (one LDS word per lane, two compares): an entry counts for
        // this wave once it has left the window of the wave's last row, and needs no mask once it has left the window
        // of the first; the filler positions of a ragged last tile never do
        const int pv = pos_lds[t & 1][lane];
        if (__builtin_amdgcn_ballot_w64(pv <= r_hi - window) != 0ull)
          mode = __builtin_amdgcn_ballot_w64(pv > r0 - window) == 0ull ? 0 : 2;
      }
    }
    mode = __builtin_amdgcn_readfirstlane(mode);
    if (mode >= 0) compute(mode, buf, pos_lds[t & 1], jt);
  };
  if (tid == 0) redo_flag = 0;
#pragma unroll 1
  for (int pass = 0; pass < 2; ++pass) {
    TR regs;
    load_tile(0, regs);
    store_tile(0, regs);
    if (n_tiles > 1) load_tile(1, regs);
    for (int t = 0; t < n_tiles; ++t) step(t, regs);
    if (exact_pass) break;
    // did a row's reference value fall so far below its scores that its sums left the range?
    bool bad = false;
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) bad = bad || !(l_part[qb] <= kBig);
    if (__builtin_amdgcn_ballot_w64(bad) != 0ull && lane == 0) redo_flag = 1;
    __syncthreads();  // also: tile buffers are free
    if (redo_flag == 0) break;
    exact_pass = true;
    reset_rows();
  }

  // ---- epilogue: normalise, stage through LDS, store rows coalesced -------------------------------------------
  __syncthreads();  // tile buffers are free
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    const float l_row = pair_sum(l_part[qb]);
    const float inv = 1.0f / l_row;
    if (lse != nullptr && hb == 0) {
      // natural-log normaliser of the scaled scores (m_run is kept in the base-2 domain); wanted by a backward pass
      const int row = (HW == 1 ? 32 * QB * wv : 0) + 32 * qb + ql;
      if (i0 + row < n) lse[(int64_t)hq * lse_stride + lo_q + i0 + row - q_begin] = (m_run[qb] + __log2f(l_row)) * 0.6931471805599453f;
    }
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
    // staging row = 32*QB*wave + position block: with HW = 1 all rows are positions of one head, with HW = 4 the
    // wave index is the head inside the group
    bf16_t* obase = out + ((int64_t)(lo_q + i0 - q_begin) * Hq + unit * HW) * D;
    const int64_t orow_stride = (int64_t)Hq * D;
#pragma unroll
    for (int p = 0; p < BM / G::RPP; ++p) {
      const int row = p * G::RPP + k_row;
      const int prow = HW == 1 ? row : row % (32 * QB), hd = HW == 1 ? 0 : row / (32 * QB);
      if (i0 + prow < n)
        *reinterpret_cast<u32x4*>(obase + prow * orow_stride + hd * D + k_piece * 8) =
            *reinterpret_cast<const u32x4*>(lds + row * G::OS + k_piece * 8);
    }
  }
}

template <int D, int QB, int HW>
hipError_t run(const ltea_cfg& cfg, const void* q, int64_t q_st, int64_t q_sh, const void* k, const void* v,
               int64_t kv_st, int64_t kv_sh, const SeqView& sv, const ltea_cache& c, void* out,
               const int32_t* kv_start, const int32_t* kv_len, float* lse, hipStream_t stream) {
  constexpr int BMQ = Geo<D, QB>::BM / HW;
  const float scale = cfg.softmax_scale > 0.f ? cfg.softmax_scale : 1.0f / sqrtf((float)cfg.D);
  const int64_t tiles_upper = (sv.total_tokens + BMQ - 1) / BMQ + sv.n_seqs;
  const int64_t n_work = tiles_upper * (cfg.Hq / HW);
  const int64_t grid = (n_work + 7) / 8 * 8;
  hipLaunchKernelGGL((attention_mfma_kernel<D, QB, HW>), dim3((unsigned)grid), dim3(kThreads), 0, stream,
                     static_cast<const bf16_t*>(q), q_st, q_sh, static_cast<const bf16_t*>(k),
                     static_cast<const bf16_t*>(v), kv_st, kv_sh, sv.cu_seqlens, sv.n_seqs, (int)tiles_upper,
                     (int)n_work, cfg.Hq, cfg.Hkv, cfg.window, cfg.budget, scale * 1.4426950408889634f,
                     static_cast<const bf16_t*>(c.k_ret), static_cast<const bf16_t*>(c.v_ret), c.ret_pos, c.ret_count,
                     static_cast<bf16_t*>(out), kv_start, kv_len, lse, sv.total_tokens);
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
                                 void* out, hipStream_t stream, const int32_t* kv_start, const int32_t* kv_len,
                                 float* lse) {
  if (sv.total_tokens == 0) return hipSuccess;
  // grouped-query shapes with a multiple of four query heads per KV head: one query head per wave (see the kernel)
  const bool by_head = (cfg.Hq / cfg.Hkv) % 4 == 0;
  if (cfg.D == 64)
    return by_head ? run<64, 1, 4>(cfg, q, q_st, q_sh, k, v, kv_st, kv_sh, sv, c, out, kv_start, kv_len, lse, stream)
                   : run<64, 1, 1>(cfg, q, q_st, q_sh, k, v, kv_st, kv_sh, sv, c, out, kv_start, kv_len, lse, stream);
  return by_head ? run<128, 1, 4>(cfg, q, q_st, q_sh, k, v, kv_st, kv_sh, sv, c, out, kv_start, kv_len, lse, stream)
                 : run<128, 1, 1>(cfg, q, q_st, q_sh, k, v, kv_st, kv_sh, sv, c, out, kv_start, kv_len, lse, stream);
}

}  // namespace ltea
