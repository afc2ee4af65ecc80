// Prefill attention over window + retained set (paper Section 3.1.3) on bf16 MFMA for gfx950.
//
// Flash-attention-style tiling, two stages per query tile as in the paper's description: stage 1 walks
// 64-key tiles of the original K/V inside the tile's window range, stage 2 walks 64-slot tiles of the
// compact retained segment with a per-row mask "position <= i - window" (so entries still inside a
// query's window are never counted twice).  Tiles wholly outside a wave's window range are skipped.
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
// V^T operand be read as one 16-byte LDS load.  V is transposed on its way into LDS.
#include "ltea_common.h"
#include "ltea_kernels.h"

namespace ltea {
namespace {

constexpr int BM = 128;  // queries per workgroup
constexpr int BN = 64;   // keys per tile
constexpr int kThreads = 256;

// Row of the K tile (within a block of 32) that MFMA row m must carry so that accumulator register r of
// lane half hb holds key 16*(r/8) + 8*hb + r%8: swap bits 2 and 3 of m.
__device__ __forceinline__ int key_row_of_mfma_row(int m) { return (m & 0x13) | ((m & 0x08) >> 1) | ((m & 0x04) << 1); }

template <int D> struct TileRegs {
  static constexpr int PPR = D / 8;                 // 16-byte pieces per K row
  static constexpr int RPP = kThreads / PPR;        // K rows per pass
  static constexpr int KPASS = BN / RPP;            // passes over the K tile
  static constexpr int CPT = D / 16;                // V columns per thread (4 keys x CPT columns)
  u32x4 k[KPASS];
  uint32_t v[4][CPT / 2];
  int pos;
};

template <int D>
__global__ void __launch_bounds__(kThreads)
attention_mfma_kernel(const bf16_t* __restrict__ q, int64_t q_st, int64_t q_sh, const bf16_t* __restrict__ k,
                      const bf16_t* __restrict__ v, int64_t kv_st, int64_t kv_sh, const int32_t* __restrict__ cu,
                      int n_seqs, int tiles_upper, int n_work, int Hq, int Hkv, int window, int budget,
                      float scale_log2e, const bf16_t* __restrict__ k_ret, const bf16_t* __restrict__ v_ret,
                      const int32_t* __restrict__ ret_pos, const int32_t* __restrict__ ret_count,
                      bf16_t* __restrict__ out) {
  using TR = TileRegs<D>;
  constexpr int KS = D + 8;    // K tile row stride (elements): 16-byte pad keeps ds_read_b128 conflict-free
  constexpr int VS = BN + 8;   // V^T tile row stride (elements)
  __shared__ __align__(16) bf16_t k_lds[BN * KS];
  __shared__ __align__(16) bf16_t vt_lds[D * VS];
  __shared__ int pos_lds[BN];

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

  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
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
  const int n_tiles = n_win_tiles + n_ret_tiles;

  const bf16_t* kbase = k + lo * kv_st + (int64_t)h * kv_sh;
  const bf16_t* vbase = v + lo * kv_st + (int64_t)h * kv_sh;
  const bf16_t* krbase = k_ret + head * budget * D;
  const bf16_t* vrbase = v_ret + head * budget * D;
  const int32_t* prbase = ret_pos + head * budget;

  const int k_piece = tid % TR::PPR, k_row = tid / TR::PPR;
  const int v_g = tid % 16, v_kg = tid / 16;

  auto load_tile = [&](int t, TR& R) {
    const bool is_ret = t >= n_win_tiles;
    const int base = is_ret ? (t - n_win_tiles) * BN : jt0 + t * BN;
    const int last = is_ret ? cnt - 1 : n - 1;
#pragma unroll
    for (int p = 0; p < TR::KPASS; ++p) {
      int idx = base + p * TR::RPP + k_row;
      idx = idx < last ? idx : last;
      const bf16_t* src = is_ret ? krbase + (int64_t)idx * D : kbase + (int64_t)idx * kv_st;
      R.k[p] = *reinterpret_cast<const u32x4*>(src + k_piece * 8);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      int idx = base + 4 * v_kg + i;
      idx = idx < last ? idx : last;
      const bf16_t* src = (is_ret ? vrbase + (int64_t)idx * D : vbase + (int64_t)idx * kv_st) + v_g * TR::CPT;
      if constexpr (TR::CPT == 8) {
        const u32x4 x = *reinterpret_cast<const u32x4*>(src);
        R.v[i][0] = x[0]; R.v[i][1] = x[1]; R.v[i][2] = x[2]; R.v[i][3] = x[3];
      } else {
        const u32x2 x = *reinterpret_cast<const u32x2*>(src);
        R.v[i][0] = x[0]; R.v[i][1] = x[1];
      }
    }
    R.pos = 0x7FFFFFFF;
    if (is_ret && tid < BN && base + tid < cnt) R.pos = prbase[base + tid];
  };

  auto store_tile = [&](int t, const TR& R) {
#pragma unroll
    for (int p = 0; p < TR::KPASS; ++p)
      *reinterpret_cast<u32x4*>(&k_lds[(p * TR::RPP + k_row) * KS + k_piece * 8]) = R.k[p];
    // transpose 4 keys x CPT columns: column c of keys 4*v_kg .. +3 becomes 8 contiguous bytes of row c
#pragma unroll
    for (int c2 = 0; c2 < TR::CPT / 2; ++c2) {
      const uint32_t a0 = R.v[0][c2], a1 = R.v[1][c2], a2 = R.v[2][c2], a3 = R.v[3][c2];
      u32x2 even, odd;
      even[0] = (a0 & 0xFFFFu) | (a1 << 16);
      even[1] = (a2 & 0xFFFFu) | (a3 << 16);
      odd[0] = (a0 >> 16) | (a1 & 0xFFFF0000u);
      odd[1] = (a2 >> 16) | (a3 & 0xFFFF0000u);
      const int col = v_g * TR::CPT + 2 * c2;
      *reinterpret_cast<u32x2*>(&vt_lds[col * VS + 4 * v_kg]) = even;
      *reinterpret_cast<u32x2*>(&vt_lds[(col + 1) * VS + 4 * v_kg]) = odd;
    }
    if (t >= n_win_tiles && tid < BN) pos_lds[tid] = R.pos;
  };

  // ---- online softmax state (per lane = per query; the two lane halves keep separate partial sums) ------
  float m_run = -INFINITY, l_part = 0.f;
  f32x16 o[D / 32];
#pragma unroll
  for (int db = 0; db < D / 32; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[db][r] = 0.f;

  const int krow_a = key_row_of_mfma_row(ql);

  TR regs;
  load_tile(0, regs);
  for (int t = 0; t < n_tiles; ++t) {
    __syncthreads();  // everyone is done reading the previous tile
    store_tile(t, regs);
    __syncthreads();
    if (t + 1 < n_tiles) load_tile(t + 1, regs);  // in flight while this tile is computed

    const bool is_ret = t >= n_win_tiles;
    const int jt = jt0 + t * BN;  // first key position of a window tile
    bool need_mask;
    if (!is_ret) {
      // keys this wave can use at all: [r0 - window + 1, r0 + 31]
      if (jt > r0 + 31 || jt + BN - 1 < r0 - window + 1) continue;
      need_mask = !(jt + BN - 1 <= r0 && jt >= r0 + 31 - window + 1);
    } else {
      need_mask = true;
    }

    // ---- S^T = K Q^T ------------------------------------------------------------------------------------
    f32x16 sacc[2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
      for (int r = 0; r < 16; ++r) sacc[kb][r] = 0.f;
      const bf16_t* arow = &k_lds[(32 * kb + krow_a) * KS + 8 * hb];
#pragma unroll
      for (int ks = 0; ks < D / 16; ++ks) {
        const bf16x8 a = *reinterpret_cast<const bf16x8*>(arow + 16 * ks);
        sacc[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qreg[ks], sacc[kb], 0, 0, 0);
      }
    }
    // register r of block kb is key (local) 32*kb + 16*(r/8) + 8*hb + r%8
    if (need_mask) {
      if (!is_ret) {
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int j = jt + 32 * kb + 16 * (r / 8) + 8 * hb + (r % 8);
            const bool ok = (j <= qi) && (j > qi - window) && (j < n);
            sacc[kb][r] = ok ? sacc[kb][r] : -INFINITY;
          }
      } else {
        const int lim = qi - window;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int p = pos_lds[32 * kb + 16 * (r / 8) + 8 * hb + (r % 8)];  // INT_MAX past ret_count
            sacc[kb][r] = (p <= lim) ? sacc[kb][r] : -INFINITY;
          }
      }
    }
    // ---- online softmax -----------------------------------------------------------------------------------
    float mx = -INFINITY;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int r = 0; r < 16; ++r) mx = fmaxf(mx, sacc[kb][r]);
    mx = fmaxf(mx, __shfl_xor(mx, 32, kWave));
    const float m_new = fmaxf(m_run, mx * scale_log2e);
    const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
    const float alpha = __builtin_amdgcn_exp2f(m_run - m_use);
    m_run = m_new;
    float psum = 0.f;
    bf16x8 pb[2][2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float p = __builtin_amdgcn_exp2f(fmaf(sacc[kb][r], scale_log2e, -m_use));
        psum += p;
        pb[kb][r / 8][r % 8] = static_cast<bf16_t>(p);
      }
    l_part = l_part * alpha + psum;
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r) o[db][r] *= alpha;
    // ---- O^T += V^T P^T -------------------------------------------------------------------------------------
#pragma unroll
    for (int db = 0; db < D / 32; ++db) {
      const bf16_t* vrow = &vt_lds[(32 * db + ql) * VS + 8 * hb];
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) {
          const bf16x8 a = *reinterpret_cast<const bf16x8*>(vrow + 32 * kb + 16 * kk);
          o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pb[kb][kk], o[db], 0, 0, 0);
        }
    }
  }

  // ---- epilogue: normalise and store --------------------------------------------------------------------------
  const float l_tot = l_part + __shfl_xor(l_part, 32, kWave);
  if (qi < n) {
    const float inv = 1.0f / l_tot;
    bf16_t* orow = out + ((lo + qi) * Hq + hq) * D;
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {
        bf16x4 w4;
#pragma unroll
        for (int e = 0; e < 4; ++e) w4[e] = static_cast<bf16_t>(o[db][4 * g4 + e] * inv);
        *reinterpret_cast<bf16x4*>(orow + 32 * db + 8 * g4 + 4 * hb) = w4;
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

bool attention_mfma_supported(const ltea_cfg& cfg) { return cfg.dtype == LTEA_BF16 && (cfg.D == 64 || cfg.D == 128); }

hipError_t launch_attention_mfma(const ltea_cfg& cfg, const void* q, int64_t q_st, int64_t q_sh, const void* k,
                                 const void* v, int64_t kv_st, int64_t kv_sh, const SeqView& sv, const ltea_cache& c,
                                 void* out, hipStream_t stream) {
  if (sv.total_tokens == 0) return hipSuccess;
  return cfg.D == 64 ? run<64>(cfg, q, q_st, q_sh, k, v, kv_st, kv_sh, sv, c, out, stream)
                     : run<128>(cfg, q, q_st, q_sh, k, v, kv_st, kv_sh, sv, c, out, stream);
}

}  // namespace ltea
