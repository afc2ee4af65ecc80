// Prefill attention over window + retained set (paper Section 3.1.3) on bf16 MFMA for gfx950.
//
// Flash-attention-style tiling, two stages per query tile as in the paper's description: stage 1 walks
// 64-key tiles of the original K/V inside the tile's window range, stage 2 walks 64-slot tiles of the
// compact retained segment with a per-row mask "position <= i - window" (so entries still inside a
// query's window are never counted twice).  Tiles wholly outside a wave's window range are skipped and
// only tiles that straddle a window edge, the causal diagonal or the sequence end pay for masking.
//
// Work split: one workgroup = 128 consecutive queries of one (sequence, query head); 4 waves x 32 queries.
// MFMA shapes (v_mfma_f32_32x32x16_bf16, wave64):
//   S^T[key, query] = K[key, :] . Q[query, :]   A = K tile rows from LDS, B = Q fragment held in registers
//   O^T[d, query]  += V^T[d, key] . P^T[key, query]   A = V^T tile from LDS, B = P^T straight from S^T's
//                                                     accumulator registers (no shuffle, no LDS round trip)
// In the 32x32 accumulator layout a lane owns one query column, so the online-softmax statistics are
// per-lane scalars (the two lanes sharing a query exchange one value per tile).  The contraction index of
// the second product is the key index; the rows of the K tile are fed to the first MFMA in a permuted
// order so that each lane's eight P values per MFMA are eight consecutive keys, which is what lets the
// V^T operand be read as one 16-byte LDS load.  V is transposed on its way into LDS (4 keys x 8 columns
// per thread, XOR-swizzled so that both the transposing stores and the operand loads spread over all banks).
// The running maximum is only raised when a tile exceeds it by more than 2^8 (the result is independent
// of the stabiliser), which keeps the accumulator rescale off the common path.
#include <type_traits>

#include "ltea_common.h"
#include "ltea_kernels.h"

namespace ltea {
namespace {

constexpr int BM = 128;  // queries per workgroup
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

template <int D> struct Geo {
  static constexpr int KS = D + 8;              // K tile row stride (elements); 16-byte pad
  static constexpr int VS = BN + 8;             // V^T tile row stride (elements)
  static constexpr int PPR = D / 8;             // 16-byte pieces per K row
  static constexpr int RPP = kThreads / PPR;    // K rows per pass
  static constexpr int KPASS = BN / RPP;        // passes over the K tile
  static constexpr int CPT = D / 16;            // V columns per thread (4 keys x CPT columns)
  static constexpr int OS = D + 8;              // epilogue staging row stride (elements)
};

template <int D> struct TileRegs {
  u32x4 k[Geo<D>::KPASS];
  uint32_t v[4][Geo<D>::CPT / 2];
  int pos;
};

template <int D>
__global__ void __launch_bounds__(kThreads, 2)
attention_mfma_kernel(const bf16_t* __restrict__ q, int64_t q_st, int64_t q_sh, const bf16_t* __restrict__ k,
                      const bf16_t* __restrict__ v, int64_t kv_st, int64_t kv_sh, const int32_t* __restrict__ cu,
                      int n_seqs, int tiles_upper, int n_work, int Hq, int Hkv, int window, int budget,
                      float scale_log2e, const bf16_t* __restrict__ k_ret, const bf16_t* __restrict__ v_ret,
                      const int32_t* __restrict__ ret_pos, const int32_t* __restrict__ ret_count,
                      bf16_t* __restrict__ out) {
  using G = Geo<D>;
  using TR = TileRegs<D>;
  constexpr int KS = G::KS, VS = G::VS;
  constexpr int kLdsK = BN * KS, kLdsV = D * VS;
  static_assert(kLdsK + kLdsV >= BM * G::OS, "epilogue staging must fit in the tile buffers");
  __shared__ __align__(16) bf16_t lds[kLdsK + kLdsV];
  __shared__ int pos_lds[BN];
  bf16_t* k_lds = lds;
  bf16_t* vt_lds = lds + kLdsK;

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
  const int r0 = i0 + 32 * wv;          // first query row of this wave
  const int qi = r0 + ql;               // this lane's query row (may be >= n in the last tile)

  // ---- Q fragment (B operand of S^T): lane holds Q[qi][16*ks + 8*hb .. +7] ---------------------------
  bf16x8 qreg[D / 16];
  {
    const int qc = qi < n ? qi : n - 1;
    const bf16_t* qrow = q + (lo + qc) * q_st + (int64_t)hq * q_sh;
#pragma unroll
    for (int ks = 0; ks < D / 16; ++ks) qreg[ks] = *reinterpret_cast<const bf16x8*>(qrow + 16 * ks + 8 * hb);
  }

  // ---- tile schedule ------------------------------------------------------------------------------------
  const int i_last = (i0 + BM < n ? i0 + BM : n) - 1;            // last real query row of the workgroup
  const int jlo = i0 - window + 1 > 0 ? i0 - window + 1 : 0;
  const int jt0 = (jlo / BN) * BN;
  const int n_win_tiles = (i_last - jt0) / BN + 1;
  const int cnt = (budget > 0 && i_last - window >= 0) ? ret_count[head] : 0;
  const int n_ret_tiles = (cnt + BN - 1) / BN;

  // ---- per-thread load addressing: 32-bit byte offsets from a uniform base -----------------------------
  const char* kbase = reinterpret_cast<const char*>(k + lo * kv_st + (int64_t)h * kv_sh);
  const char* vbase = reinterpret_cast<const char*>(v + lo * kv_st + (int64_t)h * kv_sh);
  const char* krbase = reinterpret_cast<const char*>(k_ret + head * budget * D);
  const char* vrbase = reinterpret_cast<const char*>(v_ret + head * budget * D);
  const int32_t* prbase = ret_pos + head * budget;
  const uint32_t row_bytes = (uint32_t)kv_st * 2u;
  const int k_piece = tid % G::PPR, k_row = tid / G::PPR;
  const int v_g = tid % 16, v_kg = tid / 16;   // 4 keys x CPT columns per thread; columns fastest across lanes
  const uint32_t k_col = (uint32_t)k_piece * 16u, v_col = (uint32_t)(v_g * G::CPT) * 2u;
  const uint32_t k_lim = (uint32_t)(n - 1) * row_bytes + k_col, v_lim = (uint32_t)(n - 1) * row_bytes + v_col;
  const uint32_t k_loc = (uint32_t)k_row * row_bytes + k_col;          // first pass; later passes add RPP rows
  const uint32_t v_loc = (uint32_t)(4 * v_kg) * row_bytes + v_col;     // key 4*v_kg; next keys add one row each

  auto load_win = [&](int t, TR& R) {
    const uint32_t tb = (uint32_t)(jt0 + t * BN) * row_bytes;
#pragma unroll
    for (int p = 0; p < G::KPASS; ++p) {
      uint32_t off = tb + k_loc + (uint32_t)(p * G::RPP) * row_bytes;
      off = off < k_lim ? off : k_lim;   // rows past the sequence end re-read its last row (masked later)
      R.k[p] = *reinterpret_cast<const u32x4*>(kbase + off);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      uint32_t off = tb + v_loc + (uint32_t)i * row_bytes;
      off = off < v_lim ? off : v_lim;
      if constexpr (G::CPT == 8) {
        const u32x4 x = *reinterpret_cast<const u32x4*>(vbase + off);
        R.v[i][0] = x[0]; R.v[i][1] = x[1]; R.v[i][2] = x[2]; R.v[i][3] = x[3];
      } else {
        const u32x2 x = *reinterpret_cast<const u32x2*>(vbase + off);
        R.v[i][0] = x[0]; R.v[i][1] = x[1];
      }
    }
  };
  auto load_ret = [&](int t, TR& R) {
    const int base = t * BN;
#pragma unroll
    for (int p = 0; p < G::KPASS; ++p) {
      int idx = base + p * G::RPP + k_row;
      idx = idx < cnt - 1 ? idx : cnt - 1;
      R.k[p] = *reinterpret_cast<const u32x4*>(krbase + (uint32_t)idx * (uint32_t)(D * 2) + k_col);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      int idx = base + 4 * v_kg + i;
      idx = idx < cnt - 1 ? idx : cnt - 1;
      const char* src = vrbase + (uint32_t)idx * (uint32_t)(D * 2) + v_col;
      if constexpr (G::CPT == 8) {
        const u32x4 x = *reinterpret_cast<const u32x4*>(src);
        R.v[i][0] = x[0]; R.v[i][1] = x[1]; R.v[i][2] = x[2]; R.v[i][3] = x[3];
      } else {
        const u32x2 x = *reinterpret_cast<const u32x2*>(src);
        R.v[i][0] = x[0]; R.v[i][1] = x[1];
      }
    }
    R.pos = 0x7FFFFFFF;
    if (tid < BN && base + tid < cnt) R.pos = prbase[base + tid];
  };

  // LDS store addresses. V^T rows are d, columns keys; the 16-byte column chunk index is XOR-ed with
  // 2*((d >> 4) & 3) on both the store and the load side.
  bf16_t* k_st_ptr = k_lds + k_row * KS + k_piece * 8;
  const int v_d0 = v_g * G::CPT;
  bf16_t* v_st_ptr = vt_lds + v_d0 * VS + ((4 * v_kg) ^ (16 * ((v_d0 >> 4) & 3)));
  auto store_tile = [&](const TR& R, bool with_pos) {
#pragma unroll
    for (int p = 0; p < G::KPASS; ++p) *reinterpret_cast<u32x4*>(k_st_ptr + p * G::RPP * KS) = R.k[p];
#pragma unroll
    for (int c2 = 0; c2 < G::CPT / 2; ++c2) {
      const uint32_t a0 = R.v[0][c2], a1 = R.v[1][c2], a2 = R.v[2][c2], a3 = R.v[3][c2];
      u32x2 even, odd;
      even[0] = (a0 & 0xFFFFu) | (a1 << 16);
      even[1] = (a2 & 0xFFFFu) | (a3 << 16);
      odd[0] = (a0 >> 16) | (a1 & 0xFFFF0000u);
      odd[1] = (a2 >> 16) | (a3 & 0xFFFF0000u);
      *reinterpret_cast<u32x2*>(v_st_ptr + (2 * c2) * VS) = even;
      *reinterpret_cast<u32x2*>(v_st_ptr + (2 * c2 + 1) * VS) = odd;
    }
    if (with_pos && tid < BN) pos_lds[tid] = R.pos;
  };

  // operand load addresses
  const bf16_t* a_k_ptr = k_lds + key_row_of_mfma_row(ql) * KS + 8 * hb;      // + 32*kb*KS + 16*ks
  const int s4 = ql >> 4;
  const bf16_t* a_v_ptr0 = vt_lds + ql * VS + 8 * hb + 16 * (0 ^ s4);         // kk = 0
  const bf16_t* a_v_ptr1 = vt_lds + ql * VS + 8 * hb + 16 * (1 ^ s4);         // kk = 1

  // ---- online softmax state (per lane = per query; the two lane halves keep separate partial sums) ------
  float m_run = -INFINITY, l_part = 0.f;
  f32x16 o[D / 32];
#pragma unroll
  for (int db = 0; db < D / 32; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[db][r] = 0.f;

  // mode: 0 = plain, 1 = window-edge mask (keys jt..), 2 = retained mask (positions in pos_lds).
  // The 64-key tile is consumed as two 32-key halves, each with its own softmax update, so that only one
  // 32x32 score block is live at a time.
  auto compute = [&](auto mode_tag, int jt) {
    constexpr int MODE = decltype(mode_tag)::value;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
      f32x16 sacc;
#pragma unroll
      for (int r = 0; r < 16; ++r) sacc[r] = 0.f;
#pragma unroll
      for (int ks = 0; ks < D / 16; ++ks) {
        const bf16x8 a = *reinterpret_cast<const bf16x8*>(a_k_ptr + 32 * kb * KS + 16 * ks);
        sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qreg[ks], sacc, 0, 0, 0);
      }
      // register r is key (local) 32*kb + 16*(r/8) + 8*hb + r%8
      if constexpr (MODE == 1) {
        const int jl = qi - jt - 8 * hb;            // key_local_without_hb <= jl  <=> j <= qi
        const int jw = jl - window;                 // key_local_without_hb >  jw  <=> j >  qi - window
        const int jn = n - jt - 8 * hb;             // key_local_without_hb <  jn  <=> j <  n
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int c = 32 * kb + 16 * (r / 8) + (r % 8);
          const bool ok = (c <= jl) && (c > jw) && (c < jn);
          sacc[r] = ok ? sacc[r] : -INFINITY;
        }
      } else if constexpr (MODE == 2) {
        const int lim = qi - window;
#pragma unroll
        for (int r8 = 0; r8 < 2; ++r8) {
          const int* pp = &pos_lds[32 * kb + 16 * r8 + 8 * hb];
#pragma unroll
          for (int e = 0; e < 8; ++e) sacc[8 * r8 + e] = (pp[e] <= lim) ? sacc[8 * r8 + e] : -INFINITY;  // INT_MAX past ret_count
        }
      }
      // ---- online softmax with a lazily raised maximum ----------------------------------------------------
      float mx = fmaxf(sacc[0], sacc[1]);
#pragma unroll
      for (int r = 2; r < 16; r += 2) mx = fmaxf(fmaxf(mx, sacc[r]), sacc[r + 1]);
      mx = pair_max(mx);
      const float mcand = mx * scale_log2e;
      const bool grow = mcand > m_run + kLazyMax;   // true on the first visible keys (m_run = -inf)
      if (__builtin_amdgcn_ballot_w64(grow) != 0ull) {
        const float alpha = grow ? __builtin_amdgcn_exp2f(m_run - mcand) : 1.0f;
        m_run = grow ? mcand : m_run;
        l_part *= alpha;
#pragma unroll
        for (int db = 0; db < D / 32; ++db)
#pragma unroll
          for (int r = 0; r < 16; ++r) o[db][r] *= alpha;
      }
      const float m_use = (m_run == -INFINITY) ? 0.f : m_run;
      float psum0 = 0.f, psum1 = 0.f;
      bf16x8 pb[2];
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float p = __builtin_amdgcn_exp2f(fmaf(sacc[r], scale_log2e, -m_use));
        if (r & 1) psum1 += p; else psum0 += p;
        pb[r / 8][r % 8] = static_cast<bf16_t>(p);
      }
      l_part += psum0 + psum1;
      // ---- O^T += V^T P^T -----------------------------------------------------------------------------------
#pragma unroll
      for (int db = 0; db < D / 32; ++db) {
        const int col = 32 * (kb ^ (db & 1));
        const bf16x8 a0 = *reinterpret_cast<const bf16x8*>(a_v_ptr0 + 32 * db * VS + col);
        o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, pb[0], o[db], 0, 0, 0);
        const bf16x8 a1 = *reinterpret_cast<const bf16x8*>(a_v_ptr1 + 32 * db * VS + col);
        o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, pb[1], o[db], 0, 0, 0);
      }
    }
  };

  TR regs;
  load_win(0, regs);
  // ---- stage 1: window tiles ------------------------------------------------------------------------------
  for (int t = 0; t < n_win_tiles; ++t) {
    __syncthreads();  // everyone is done reading the previous tile
    store_tile(regs, false);
    __syncthreads();
    if (t + 1 < n_win_tiles) load_win(t + 1, regs);      // in flight while this tile is computed
    else if (n_ret_tiles > 0) load_ret(0, regs);
    const int jt = jt0 + t * BN;
    // keys this wave can use at all: [r0 - window + 1, r0 + 31]
    if (jt > r0 + 31 || jt + BN - 1 < r0 - window + 1) continue;
    const bool plain = (jt + BN - 1 <= r0) && (jt >= r0 + 31 - window + 1);
    if (plain) compute(std::integral_constant<int, 0>{}, jt);
    else compute(std::integral_constant<int, 1>{}, jt);
  }
  // ---- stage 2: retained tiles ------------------------------------------------------------------------------
  for (int t = 0; t < n_ret_tiles; ++t) {
    __syncthreads();
    store_tile(regs, true);
    __syncthreads();
    if (t + 1 < n_ret_tiles) load_ret(t + 1, regs);
    compute(std::integral_constant<int, 2>{}, 0);
  }

  // ---- epilogue: normalise, stage through LDS, store rows coalesced -------------------------------------------
  const float l_tot = pair_sum(l_part);
  const float inv = 1.0f / l_tot;
  __syncthreads();  // tile buffers are free
  {
    bf16_t* orow = lds + (32 * wv + ql) * G::OS + 4 * hb;
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {
        bf16x4 w4;
#pragma unroll
        for (int e = 0; e < 4; ++e) w4[e] = static_cast<bf16_t>(o[db][4 * g4 + e] * inv);
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

template <int D>
hipError_t run(const ltea_cfg& cfg, const void* q, int64_t q_st, int64_t q_sh, const void* k, const void* v,
               int64_t kv_st, int64_t kv_sh, const SeqView& sv, const ltea_cache& c, void* out, hipStream_t stream) {
  const float scale = cfg.softmax_scale > 0.f ? cfg.softmax_scale : 1.0f / sqrtf((float)cfg.D);
  const int64_t tiles_upper = (sv.total_tokens + BM - 1) / BM + sv.n_seqs;
  const int64_t n_work = tiles_upper * cfg.Hq;
  const int64_t grid = (n_work + 7) / 8 * 8;
  hipLaunchKernelGGL(attention_mfma_kernel<D>, dim3((unsigned)grid), dim3(kThreads), 0, stream,
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
  return cfg.D == 64 ? run<64>(cfg, q, q_st, q_sh, k, v, kv_st, kv_sh, sv, c, out, stream)
                     : run<128>(cfg, q, q_st, q_sh, k, v, kv_st, kv_sh, sv, c, out, stream);
}

}  // namespace ltea
