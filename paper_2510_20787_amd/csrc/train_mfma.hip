// Training-side backward of the SWA+LTE attention on bf16 MFMA for gfx950, head dimensions 64 and 128 (paper
// Section 3.1.2: the gradients that reach Q, K, V and, through the straight-through estimator, the retention scores).
//
// Three launches on the caller's stream:
//   train_delta_mfma_kernel      delta = <dO, O> per (query, query head).
//   train_dq_far_mfma_kernel     two independent roles in one grid: the far pass of dK / dV (first, few and
//                                long-running workgroups) and dQ (fills the compute units the far pass leaves idle).
//   train_dkv_band_mfma_kernel   the band pass of dK / dV, which adds the far pass in, stores dK, dV and forms
//                                d logit and the retention counts.
//
// dQ role: one workgroup = 128 consecutive queries of one (sequence, query head), 4 waves x 32 queries, walking the
// same key tiles as the forward kernel (64-key tiles of K/V inside the window range, then 64-slot tiles of the
// compacted candidates with the per-row mask "position <= i - window").  Per 32-key block and wave
// (v_mfma_f32_32x32x16_bf16, a lane owns one query column):
//   S^T[key, query]  = K . Q^T        A = K tile rows from LDS, B = Q fragment in registers
//   dP^T[key, query] = V . dO^T       A = V tile rows from LDS, B = dO fragment in registers
//   P^T = exp2(S^T c - lse), dS^T = P^T (dP^T - delta)      per-lane scalars lse, delta (no running maximum)
//   dQ^T[d, query]  += K^T . dS^T     A = K^T through the transposing LDS load, B = dS^T straight from registers
// K is therefore staged twice per tile (padded rows for the row reads, swizzled unpadded rows for the transposing
// reads), V once.  The dK / dV roles are the mirror image with a lane owning a key column (see dkv_body).
// Two tile buffers and a register prefetch: one barrier per tile.  No floating-point atomics: the
// partial sums of the far pass go to scratch slices that the band pass adds in a fixed order.
#include "ltea_common.h"
#include "ltea_kernels.h"
#include "mfma_tiles.h"
#include "train_common.h"

namespace ltea {
namespace {

constexpr int BN = 64;          // keys (or queries) per tile
constexpr int BM = 128;         // queries (or keys) per workgroup
constexpr int kThreads = 256;

template <int D> struct Geo {
  static constexpr int KS = D + 8;       // padded row stride (elements) of tiles read row-wise
  static constexpr int VS = D;           // unpadded, chunk-swizzled row stride of tiles read through the transposing load
  static constexpr int PPR = D / 8;      // 16-byte pieces per row
  static constexpr int RPP = kThreads / PPR;
  static constexpr int KPASS = BN / RPP;
  static constexpr int OS = D + 8;       // epilogue staging stride
  static constexpr int kBufDq = 2 * BN * KS + BN * VS;        // K rows | K for transposed reads | V rows
  static constexpr int kBufDkv = 2 * BN * KS + 2 * BN * VS;   // Q rows | Q transposed | dO rows | dO transposed
  static constexpr int kBuf = kBufDkv;
};
#define LTEA_GEO(D) \
  using G_ = Geo<D>; \
  constexpr int KS = G_::KS, VS = G_::VS, PPR = G_::PPR, RPP = G_::RPP, KPASS = G_::KPASS, OS = G_::OS

template <int D> struct TileRegs {
  u32x4 a[Geo<D>::KPASS], b[Geo<D>::KPASS];
  int pos;
};

template <int D>
__device__ __forceinline__ void dq_body(const TrainArgs& A, int tiles_upper, int n_work, float scale_log2e, int block,
                                        bf16_t* lds, int* pos_lds_base, int* pos_rng_base) {
  LTEA_GEO(D);
  constexpr int kK = 0, kKt = BN * KS, kV = BN * KS + BN * VS;
  static_assert(G_::kBufDq >= BM * OS, "epilogue staging must fit in the tile buffer");

  const int per_xcd = (n_work + 7) / 8;
  const int work = (block % 8) * per_xcd + block / 8;
  if (work >= n_work) return;
  const int hq = work / tiles_upper;
  int tile, s, n, lo;
  if (!locate_tile(A.cu, A.n_seqs, BM, work - hq * tiles_upper, s, tile, lo, n)) return;
  const int Hq = A.Hq, Hkv = A.Hkv, window = A.window, budget = A.budget;
  const int h = hq / (Hq / Hkv);
  const int64_t head = (int64_t)s * Hkv + h;
  const int i0 = tile * BM;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int ql = lane & 31, hb = lane >> 5;
  const int r0 = i0 + 32 * wv;
  const int r_hi = r0 + 31;

  const bf16_t* q = static_cast<const bf16_t*>(A.q);
  const bf16_t* k = static_cast<const bf16_t*>(A.k);
  const bf16_t* v = static_cast<const bf16_t*>(A.v);
  const bf16_t* dout = static_cast<const bf16_t*>(A.dout);

  // ---- per-lane query state: Q and dO fragments (B operands), lse (base-2 domain), delta ---------------------
  const int qi = r0 + ql;
  const int qc = qi < n ? qi : n - 1;
  bf16x8 qreg[D / 16], doreg[D / 16];
  {
    const bf16_t* qrow = q + (int64_t)(lo + qc) * A.q_st + (int64_t)hq * A.q_sh;
    const bf16_t* dorow = dout + ((int64_t)(lo + qc) * Hq + hq) * D;
#pragma unroll
    for (int ks = 0; ks < D / 16; ++ks) {
      qreg[ks] = *reinterpret_cast<const bf16x8*>(qrow + 16 * ks + 8 * hb);
      doreg[ks] = *reinterpret_cast<const bf16x8*>(dorow + 16 * ks + 8 * hb);
    }
  }
  const float lse2 = A.lse[(int64_t)hq * A.total + lo + qc] * 1.4426950408889634f;
  // delta = <dO, O> of the lane's query: each lane half holds half of the row
  float dlt = 0.f;
  {
    const bf16_t* orow = static_cast<const bf16_t*>(A.out) + ((int64_t)(lo + qc) * Hq + hq) * D;
#pragma unroll
    for (int ks = 0; ks < D / 16; ++ks) {
      const bf16x8 o8 = *reinterpret_cast<const bf16x8*>(orow + 16 * ks + 8 * hb);
#pragma unroll
      for (int e = 0; e < 8; ++e) dlt = fmaf(static_cast<float>(doreg[ks][e]), static_cast<float>(o8[e]), dlt);
    }
    dlt = pair_sum(dlt);
  }

  // ---- tile schedule (as in the forward) ------------------------------------------------------------------
  const int i_last = (i0 + BM < n ? i0 + BM : n) - 1;
  const int jlo = i0 - window + 1 > 0 ? i0 - window + 1 : 0;
  const int jt0 = (jlo / BN) * BN;
  const int n_win_tiles = (i_last - jt0) / BN + 1;
  const int cnt = (budget > 0 && i_last - window >= 0) ? A.ret_count[head] : 0;
  const int n_ret_tiles = (cnt + BN - 1) / BN;
  const int n_tiles = n_win_tiles + n_ret_tiles;

  const uint32_t row_bytes = (uint32_t)A.kv_st * 2u;
  const uint32_t win_bytes = (uint32_t)(n - 1) * row_bytes + (uint32_t)(D * 2);
  const uint32_t ret_bytes = (uint32_t)cnt * (uint32_t)(D * 2);
  const auto rs_k = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t*>(k + (int64_t)lo * A.kv_st + (int64_t)h * A.kv_sh), 0, win_bytes, 0x00020000);
  const auto rs_v = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t*>(v + (int64_t)lo * A.kv_st + (int64_t)h * A.kv_sh), 0, win_bytes, 0x00020000);
  const auto rs_kr = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t*>(static_cast<const bf16_t*>(A.k_ret) + head * budget * D), 0, ret_bytes, 0x00020000);
  const auto rs_vr = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t*>(static_cast<const bf16_t*>(A.v_ret) + head * budget * D), 0, ret_bytes, 0x00020000);
  const int32_t* prbase = A.ret_pos + head * budget;
  const int k_piece = tid % PPR, k_row = tid / PPR;
  const uint32_t k_col = (uint32_t)k_piece * 16u;
  const uint32_t k_loc = (uint32_t)k_row * row_bytes + k_col;
  const uint32_t kr_loc = (uint32_t)k_row * (uint32_t)(D * 2) + k_col;

  auto load_rows = [&](const auto& rk, const auto& rv, uint32_t b0, uint32_t rb, TileRegs<D>& R) {
#pragma unroll
    for (int p = 0; p < KPASS; ++p) {
      R.a[p] = __builtin_amdgcn_raw_buffer_load_b128(rk, b0 + (uint32_t)(p * RPP) * rb, 0, 0);
      R.b[p] = __builtin_amdgcn_raw_buffer_load_b128(rv, b0 + (uint32_t)(p * RPP) * rb, 0, 0);
    }
  };
  auto load_tile = [&](int t, TileRegs<D>& R) {
    if (t < n_win_tiles) {
      load_rows(rs_k, rs_v, (uint32_t)(jt0 + t * BN) * row_bytes + k_loc, row_bytes, R);
    } else {
      const int base = (t - n_win_tiles) * BN;
      load_rows(rs_kr, rs_vr, (uint32_t)base * (uint32_t)(D * 2) + kr_loc, (uint32_t)(D * 2), R);
      R.pos = 0x7FFFFFFF;
      if (tid < BN && base + tid < cnt) R.pos = prbase[base + tid];
    }
  };
  static_assert(RPP % 4 == 0, "row passes must preserve the swizzle phase");
  const int p_st_off = k_row * KS + k_piece * 8;
  const int t_st_off = k_row * VS + (((k_piece >> 2) ^ chunk_swizzle<D>(k_row)) << 5) + (k_piece & 3) * 8;
  auto store_tile = [&](int t, const TileRegs<D>& R) {
    bf16_t* sb = lds + (t & 1) * G_::kBufDq;
#pragma unroll
    for (int p = 0; p < KPASS; ++p) {
      *reinterpret_cast<u32x4*>(sb + kK + p_st_off + p * RPP * KS) = R.a[p];
      *reinterpret_cast<u32x4*>(sb + kKt + t_st_off + p * RPP * VS) = R.a[p];
      *reinterpret_cast<u32x4*>(sb + kV + p_st_off + p * RPP * KS) = R.b[p];
    }
    if (t >= n_win_tiles && wv == 0) {
      pos_lds_base[(t & 1) * BN + lane] = R.pos;
      const int mn = wave_min_i(R.pos);
      const int mx = wave_max_i(R.pos == 0x7FFFFFFF ? (int)0x80000000 : R.pos);
      if (lane == 0) { pos_rng_base[(t & 1) * 2] = mn; pos_rng_base[(t & 1) * 2 + 1] = mx; }
    }
  };
  const bf16_t* tb = lds;            // tile buffer and position list of the tile being computed
  const int* pos_lds = pos_lds_base;

  const int a_row_off = tile_row_of_mfma_row(ql) * KS + 8 * hb;        // + 32*kb*KS + 16*ks
  const int tr_key = 8 * hb + ((lane & 15) >> 2);
  const int tr_col = 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
  const int tr_swz = chunk_swizzle<D>(tr_key);
  const int a_tr_off = kKt + tr_key * VS + tr_col;

  f32x16 acc[D / 32];
#pragma unroll
  for (int db = 0; db < D / 32; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[db][r] = 0.f;

  // mode: 0 = every pair valid, 1 = window-edge mask, 2 = mask by the candidates' positions
  auto compute = [&](const int mode, int jt) {
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
      f32x16 sc, dp;
#pragma unroll
      for (int r = 0; r < 16; ++r) { sc[r] = 0.f; dp[r] = 0.f; }
#pragma unroll
      for (int ks = 0; ks < D / 16; ++ks) {
        const bf16x8 ak = *reinterpret_cast<const bf16x8*>(tb + kK + a_row_off + 32 * kb * KS + 16 * ks);
        const bf16x8 av = *reinterpret_cast<const bf16x8*>(tb + kV + a_row_off + 32 * kb * KS + 16 * ks);
        sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ak, qreg[ks], sc, 0, 0, 0);
        dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, doreg[ks], dp, 0, 0, 0);
      }
      // register r is local key 32*kb + 16*(r/8) + 8*hb + r%8
      if (mode == 1) {
        const int shift = jt + 8 * hb;
        int c_hi = qi - shift;
        const int c_end = n - 1 - shift;
        c_hi = c_hi < c_end ? c_hi : c_end;
        int c_lo = qi - window + 1 - shift;
        const unsigned span = c_hi >= c_lo ? (unsigned)(c_hi - c_lo) : 0u;
        if (c_hi < c_lo) c_lo = 0x40000000;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int c = 32 * kb + 16 * (r / 8) + (r % 8);
          sc[r] = ((unsigned)(c - c_lo) <= span) ? sc[r] : -INFINITY;
        }
      } else if (mode == 2) {
        const int lim = qi - window;
#pragma unroll
        for (int r8 = 0; r8 < 2; ++r8) {
          const int* pp = pos_lds + 32 * kb + 16 * r8 + 8 * hb;
#pragma unroll
          for (int e = 0; e < 8; ++e) sc[8 * r8 + e] = (pp[e] <= lim) ? sc[8 * r8 + e] : -INFINITY;
        }
      }
      bf16x8 pb[2];
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float p = __builtin_amdgcn_exp2f(fmaf(sc[r], scale_log2e, -lse2));   // exp2(-inf) = 0 for masked pairs
        pb[r / 8][r % 8] = static_cast<bf16_t>(p * (dp[r] - dlt));
      }
#pragma unroll
      for (int db = 0; db < D / 32; ++db) {
        const bf16_t* ap = tb + a_tr_off + 32 * kb * VS + ((db ^ tr_swz) << 5);
        const bf16x8 a0 = load_transposed(ap, VS);
        const bf16x8 a1 = load_transposed(ap + 16 * VS, VS);
        acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, pb[0], acc[db], 0, 0, 0);
        acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, pb[1], acc[db], 0, 0, 0);
      }
    }
  };

  // tile t is computed from buffer t & 1 while tile t+1 is stored into the other buffer and tile t+2 is in flight
  TileRegs<D> regs;
  load_tile(0, regs);
  store_tile(0, regs);
  if (n_tiles > 1) load_tile(1, regs);
  for (int t = 0; t < n_tiles; ++t) {
    __syncthreads();                 // tile t is in LDS; everyone is done with tile t-1 (its buffer is written next)
    if (t + 1 < n_tiles) store_tile(t + 1, regs);
    if (t + 2 < n_tiles) load_tile(t + 2, regs);
    tb = lds + (t & 1) * G_::kBufDq;
    pos_lds = pos_lds_base + (t & 1) * BN;
    int mode = -1, jt = 0;
    if (r0 < n) {
      if (t < n_win_tiles) {
        jt = jt0 + t * BN;
        if (!(jt > r_hi || jt + BN - 1 < r0 - window + 1))
          mode = ((jt + BN - 1 <= r0) && (jt >= r_hi - window + 1)) ? 0 : 1;
      } else {
        const int pmin = pos_rng_base[(t & 1) * 2], pmax = pos_rng_base[(t & 1) * 2 + 1];
        if (pmin <= r_hi - window) {
          const bool full = (t - n_win_tiles + 1) * BN <= cnt;
          mode = (full && pmax <= r0 - window) ? 0 : 2;
        }
      }
    }
    mode = __builtin_amdgcn_readfirstlane(mode);
    if (mode == 0) compute(0, jt);
    else if (mode == 1) compute(1, jt);
    else if (mode == 2) compute(2, jt);
  }

  // ---- epilogue: dQ = scale * acc, staged through LDS, rows stored coalesced ---------------------------------
  __syncthreads();
  {
    bf16_t* orow = lds + (32 * wv + ql) * OS + 4 * hb;
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {
        bf16x4 w4;
#pragma unroll
        for (int e = 0; e < 4; ++e) w4[e] = static_cast<bf16_t>(acc[db][4 * g4 + e] * A.scale);
        *reinterpret_cast<bf16x4*>(orow + 32 * db + 8 * g4) = w4;
      }
  }
  __syncthreads();
  {
    bf16_t* obase = static_cast<bf16_t*>(A.dq) + ((int64_t)(lo + i0) * Hq + hq) * D;
    const int64_t orow_stride = (int64_t)Hq * D;
#pragma unroll
    for (int p = 0; p < BM / RPP; ++p) {
      const int row = p * RPP + k_row;
      if (i0 + row < n)
        *reinterpret_cast<u32x4*>(obase + row * orow_stride + k_piece * 8) =
            *reinterpret_cast<const u32x4*>(lds + row * OS + k_piece * 8);
    }
  }
}



template <int D> struct QTileRegs {
  u32x4 a[Geo<D>::KPASS], b[Geo<D>::KPASS];
  float stat;     // threads 0..63: lse (base-2 domain) of a query of the tile, threads 64..127: its delta
};

// train_dkv_mfma_kernel<FAR>: one workgroup = 128 keys of one (sequence, KV head), 4 waves x 32 keys; a lane owns one
// key column.  It walks 64-query tiles of every query head of the group that can see its keys:
//   S[query, key]  = Q . K^T          A = Q tile rows from LDS, B = K fragment in registers
//   dP[query, key] = dO . V^T         A = dO tile rows from LDS, B = V fragment in registers
//   P = exp2(S c - lse[query]), dS = P (dP - delta[query])      lse, delta per row, read from LDS
//   dV^T[d, key] += dO^T . P          A = dO^T through the transposing LDS load, B = P from registers
//   dK^T[d, key] += Q^T . dS          A = Q^T through the transposing LDS load, B = dS from registers
// FAR = false ("band"): the keys are 128 consecutive positions, seen by the queries j .. j+window-1; the epilogue adds
// what the FAR pass left for keys that are candidates, rounds and stores dK, dV, and forms d logit and the counts.
// FAR = true: the keys are 128 consecutive entries of the compacted candidates (positions ascending), seen by the
// queries from position + window on; the fp32 sums go to a scratch array indexed like the compact segment.
template <int D, bool FAR>
__device__ __forceinline__ void dkv_body(const TrainArgs& A, int tiles_upper, float scale_log2e, float* far_dk,
                                         float* far_dv, int block, bf16_t* lds, float* stat_base) {
  LTEA_GEO(D);
  constexpr int kQ = 0, kQt = BN * KS, kO = BN * KS + BN * VS, kOt = 2 * BN * KS + BN * VS;
  static_assert(G_::kBufDkv >= BM * OS, "epilogue staging must fit in the tile buffer");

  const int Hq = A.Hq, Hkv = A.Hkv, window = A.window, cap = A.budget;
  const int G = Hq / Hkv;
  int s, n, lo, h, j0 = 0, r_base = 0, cnt = 0;
  int chunk = 0;                          // FAR: which share of the query tiles this workgroup walks
  if (FAR) {
    // one workgroup per (128 compact entries, share of the query range): A.far_chunks shares of equal length keep
    // the workgroups short and alike; their partial sums go to one scratch slice each, which the band pass adds up
    // in a fixed order
    // The workgroups of one (head, share) read the same Q and dO tiles: order them so that they are neighbours, and
    // give each XCD a contiguous range of that order (workgroups are dealt round-robin to the 8 XCDs).
    const int per_head = (A.max_seqlen + BM - 1) / BM;
    const int n_far = A.n_seqs * Hkv * A.far_chunks * per_head;
    const int per_xcd = (n_far + 7) / 8;
    const int work = (block % 8) * per_xcd + block / 8;
    if (work >= n_far) return;            // padding workgroups of the combined launch
    const int rest = work / per_head;
    chunk = rest % A.far_chunks;
    const int hd = rest / A.far_chunks;
    r_base = (work - rest * per_head) * BM;
    s = hd / Hkv;
    h = hd - s * Hkv;
    cnt = A.ret_count[hd];
    if (r_base >= cnt) return;
    lo = A.cu[s];
    n = A.cu[s + 1] - lo;
  } else {
    // Workgroups are dealt round-robin to the 8 XCDs; give each XCD a contiguous range of key tiles so that
    // neighbouring tiles of one head (which walk mostly the same Q and dO tiles) meet in the same L2.
    const int n_work = tiles_upper * Hkv;
    const int per_xcd = (n_work + 7) / 8;
    const int work = (block % 8) * per_xcd + block / 8;
    if (work >= n_work) return;
    h = work / tiles_upper;
    int tile;
    if (!locate_tile(A.cu, A.n_seqs, BM, work - h * tiles_upper, s, tile, lo, n)) return;
    j0 = tile * BM;
  }
  const int64_t head = (int64_t)s * Hkv + h;
  const int32_t* rp = A.ret_pos + head * cap;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int ql = lane & 31, hb = lane >> 5;
  const bf16_t* q = static_cast<const bf16_t*>(A.q);
  const bf16_t* dout = static_cast<const bf16_t*>(A.dout);

  // ---- this lane's key: its K / V fragments and the range of queries [q_lo, q_hi) that saw it -----------------
  const int kloc = 32 * wv + ql;          // key index inside the workgroup
  int q_lo = 0, q_hi = 0, jpos = 0;
  const bf16_t *krow, *vrow;
  bool key_ok;
  if (FAR) {
    const int r = r_base + kloc;
    key_ok = r < cnt;
    const int rc = key_ok ? r : cnt - 1;
    jpos = rp[rc];
    krow = static_cast<const bf16_t*>(A.k_ret) + (head * cap + rc) * D;
    vrow = static_cast<const bf16_t*>(A.v_ret) + (head * cap + rc) * D;
    if (key_ok) { q_lo = jpos + window; q_hi = n; }
  } else {
    const int j = j0 + kloc;
    key_ok = j < n;
    jpos = key_ok ? j : n - 1;
    krow = static_cast<const bf16_t*>(A.k) + (int64_t)(lo + jpos) * A.kv_st + (int64_t)h * A.kv_sh;
    vrow = static_cast<const bf16_t*>(A.v) + (int64_t)(lo + jpos) * A.kv_st + (int64_t)h * A.kv_sh;
    if (key_ok) { q_lo = j; q_hi = j + window < n ? j + window : n; }
  }
  const unsigned q_span = (unsigned)(q_hi - q_lo);     // 0 for lanes without a key
  bf16x8 kreg[D / 16], vreg[D / 16];
#pragma unroll
  for (int ks = 0; ks < D / 16; ++ks) {
    kreg[ks] = *reinterpret_cast<const bf16x8*>(krow + 16 * ks + 8 * hb);
    vreg[ks] = *reinterpret_cast<const bf16x8*>(vrow + 16 * ks + 8 * hb);
  }

  // ---- query tiles the workgroup has to visit (the same for every query head of the group) --------------------
  int qt_first, qt_last;
  const int chunk_tiles = ((n + BN - 1) / BN + A.far_chunks - 1) / A.far_chunks;   // query tiles per share
  if (FAR) {
    qt_first = (rp[r_base] + window) / BN;            // positions ascend: the first entry is seen first
    qt_last = (n - 1) / BN;
    qt_first = qt_first > chunk * chunk_tiles ? qt_first : chunk * chunk_tiles;
    qt_last = qt_last < (chunk + 1) * chunk_tiles - 1 ? qt_last : (chunk + 1) * chunk_tiles - 1;
    if (qt_first > qt_last) return;                   // this share lies before the entries' first query: nothing to add
  } else {
    qt_first = j0 / BN;
    const int last_key = (j0 + BM < n ? j0 + BM : n) - 1;
    const int last_q = last_key + window - 1 < n - 1 ? last_key + window - 1 : n - 1;
    qt_last = last_q / BN;
  }
  const int n_qt = qt_last - qt_first + 1;
  const int n_iter = n_qt * G;

  const uint32_t q_row_bytes = (uint32_t)A.q_st * 2u, o_row_bytes = (uint32_t)(Hq * D) * 2u;
  const uint32_t q_bytes = (uint32_t)(n - 1) * q_row_bytes + (uint32_t)(D * 2);
  const uint32_t o_bytes = (uint32_t)(n - 1) * o_row_bytes + (uint32_t)(D * 2);
  const int k_piece = tid % PPR, k_row = tid / PPR;
  auto load_tile = [&](int it, QTileRegs<D>& R) {
    const int g = it / n_qt, t = it - g * n_qt;
    const int hq = h * G + g;
    const int qt = (qt_first + t) * BN;
    const auto rs_q = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t*>(q + (int64_t)lo * A.q_st + (int64_t)hq * A.q_sh), 0, q_bytes, 0x00020000);
    const auto rs_o = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t*>(dout + ((int64_t)lo * Hq + hq) * D), 0, o_bytes, 0x00020000);
#pragma unroll
    for (int p = 0; p < KPASS; ++p) {
      const uint32_t row = (uint32_t)(qt + k_row + p * RPP);
      R.a[p] = __builtin_amdgcn_raw_buffer_load_b128(rs_q, row * q_row_bytes + (uint32_t)k_piece * 16u, 0, 0);
      R.b[p] = __builtin_amdgcn_raw_buffer_load_b128(rs_o, row * o_row_bytes + (uint32_t)k_piece * 16u, 0, 0);
    }
    if (tid < 2 * BN) {
      const int qrow = qt + (tid & (BN - 1));
      const int qc = qrow < n ? qrow : n - 1;
      const int64_t idx = (int64_t)hq * A.total + lo + qc;
      R.stat = tid < BN ? A.lse[idx] * 1.4426950408889634f : A.delta[idx];
    }
  };
  static_assert(RPP % 4 == 0, "row passes must preserve the swizzle phase");
  const int p_st_off = k_row * KS + k_piece * 8;
  const int t_st_off = k_row * VS + (((k_piece >> 2) ^ chunk_swizzle<D>(k_row)) << 5) + (k_piece & 3) * 8;
  auto store_tile = [&](int it, const QTileRegs<D>& R) {
    bf16_t* sb = lds + (it & 1) * G_::kBufDkv;
#pragma unroll
    for (int p = 0; p < KPASS; ++p) {
      *reinterpret_cast<u32x4*>(sb + kQ + p_st_off + p * RPP * KS) = R.a[p];
      *reinterpret_cast<u32x4*>(sb + kQt + t_st_off + p * RPP * VS) = R.a[p];
      *reinterpret_cast<u32x4*>(sb + kO + p_st_off + p * RPP * KS) = R.b[p];
      *reinterpret_cast<u32x4*>(sb + kOt + t_st_off + p * RPP * VS) = R.b[p];
    }
    if (tid < 2 * BN) stat_base[(it & 1) * 2 * BN + tid] = R.stat;     // [lse of the 64 queries | their delta]
  };
  const bf16_t* tb = lds;            // tile buffer and row statistics of the tile being computed
  const float *lse_lds = stat_base, *dlt_lds = stat_base + BN;

  const int a_row_off = tile_row_of_mfma_row(ql) * KS + 8 * hb;        // + 32*qb*KS + 16*ks
  const int tr_row = 8 * hb + ((lane & 15) >> 2);
  const int tr_col = 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
  const int tr_swz = chunk_swizzle<D>(tr_row);
  const int a_tr_off = tr_row * VS + tr_col;

  f32x16 dva[D / 32], dka[D / 32];
#pragma unroll
  for (int db = 0; db < D / 32; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) { dva[db][r] = 0.f; dka[db][r] = 0.f; }

  auto compute = [&](const bool masked, int qt) {
#pragma unroll 1
    for (int qb = 0; qb < 2; ++qb) {
      f32x16 sc, dp;
#pragma unroll
      for (int r = 0; r < 16; ++r) { sc[r] = 0.f; dp[r] = 0.f; }
#pragma unroll
      for (int ks = 0; ks < D / 16; ++ks) {
        const bf16x8 aq = *reinterpret_cast<const bf16x8*>(tb + kQ + a_row_off + 32 * qb * KS + 16 * ks);
        const bf16x8 ao = *reinterpret_cast<const bf16x8*>(tb + kO + a_row_off + 32 * qb * KS + 16 * ks);
        sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(aq, kreg[ks], sc, 0, 0, 0);
        dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ao, vreg[ks], dp, 0, 0, 0);
      }
      // register r is the tile's query 32*qb + 16*(r/8) + 8*hb + r%8
      bf16x8 pp[2], ps[2];
#pragma unroll
      for (int r8 = 0; r8 < 2; ++r8) {
        const int row0 = 32 * qb + 16 * r8 + 8 * hb;
        const f32x4 l0 = *reinterpret_cast<const f32x4*>(lse_lds + row0), l1 = *reinterpret_cast<const f32x4*>(lse_lds + row0 + 4);
        const f32x4 d0 = *reinterpret_cast<const f32x4*>(dlt_lds + row0), d1 = *reinterpret_cast<const f32x4*>(dlt_lds + row0 + 4);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float l = e < 4 ? l0[e] : l1[e - 4];
          const float dl = e < 4 ? d0[e] : d1[e - 4];
          float p = __builtin_amdgcn_exp2f(fmaf(sc[8 * r8 + e], scale_log2e, -l));
          if (masked) p = ((unsigned)(qt + row0 + e - q_lo) < q_span) ? p : 0.f;
          pp[r8][e] = static_cast<bf16_t>(p);
          ps[r8][e] = static_cast<bf16_t>(p * (dp[8 * r8 + e] - dl));
        }
      }
#pragma unroll
      for (int db = 0; db < D / 32; ++db) {
        const bf16_t* ao = tb + kOt + a_tr_off + 32 * qb * VS + ((db ^ tr_swz) << 5);
        const bf16_t* aq = tb + kQt + a_tr_off + 32 * qb * VS + ((db ^ tr_swz) << 5);
        const bf16x8 o0 = load_transposed(ao, VS), o1 = load_transposed(ao + 16 * VS, VS);
        const bf16x8 q0 = load_transposed(aq, VS), q1 = load_transposed(aq + 16 * VS, VS);
        dva[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(o0, pp[0], dva[db], 0, 0, 0);
        dva[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(o1, pp[1], dva[db], 0, 0, 0);
        dka[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(q0, ps[0], dka[db], 0, 0, 0);
        dka[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(q1, ps[1], dka[db], 0, 0, 0);
      }
    }
  };

  // tile `it` is computed from buffer it & 1 while the next one is stored into the other and the one after is in flight
  QTileRegs<D> regs;
  load_tile(0, regs);
  store_tile(0, regs);
  if (n_iter > 1) load_tile(1, regs);
  for (int it = 0; it < n_iter; ++it) {
    __syncthreads();
    if (it + 1 < n_iter) store_tile(it + 1, regs);
    if (it + 2 < n_iter) load_tile(it + 2, regs);
    tb = lds + (it & 1) * G_::kBufDkv;
    lse_lds = stat_base + (it & 1) * 2 * BN;
    dlt_lds = lse_lds + BN;
    const int t = it % n_qt;
    const int qt = (qt_first + t) * BN;
    // does any key of this wave see a query of the tile, and do all of them see all of it?
    const bool touches = q_span != 0u && q_lo < qt + BN && q_hi > qt;
    const bool covers = q_span != 0u && q_lo <= qt && q_hi >= qt + BN;
    if (__builtin_amdgcn_ballot_w64(touches) == 0ull) continue;
    if (__builtin_amdgcn_ballot_w64(!covers) == 0ull) compute(false, qt);
    else compute(true, qt);
  }

  // ---- epilogue: accumulator register r of block db is feature d = 32*db + 8*(r/4) + 4*hb + r%4 of the lane's key ---
  if (FAR) {
    if (key_ok) {
      const int64_t slice = (int64_t)chunk * A.n_seqs * Hkv + head;
      float* fk = far_dk + (slice * cap + r_base + kloc) * D + 4 * hb;
      float* fv = far_dv + (slice * cap + r_base + kloc) * D + 4 * hb;
#pragma unroll
      for (int db = 0; db < D / 32; ++db)
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4) {
          f32x4 a, b;
#pragma unroll
          for (int e = 0; e < 4; ++e) { a[e] = dka[db][4 * g4 + e] * A.scale; b[e] = dva[db][4 * g4 + e]; }
          *reinterpret_cast<f32x4*>(fk + 32 * db + 8 * g4) = a;
          *reinterpret_cast<f32x4*>(fv + 32 * db + 8 * g4) = b;
        }
    }
    return;
  }
  // band: add the far part of candidate keys (their compact index by binary search over the ascending positions)
  int ridx = -1;
  if (key_ok && cap > 0) {
    int a = 0, b = A.ret_count[head];
    while (a < b) {
      const int mid = (a + b) >> 1;
      if (rp[mid] < jpos) a = mid + 1; else b = mid;
    }
    if (a < A.ret_count[head] && rp[a] == jpos) ridx = a;
  }
  // the shares of the query range in which the far pass wrote something for this entry's group of 128
  int c_first = 0, c_last = -1;
  if (ridx >= 0) {
    c_first = ((rp[ridx / BM * BM] + window) / BN) / chunk_tiles;
    c_last = ((n - 1) / BN) / chunk_tiles;
  }
  float ste = 0.f;
#pragma unroll
  for (int db = 0; db < D / 32; ++db)
#pragma unroll
    for (int g4 = 0; g4 < 4; ++g4) {
      const int d0 = 32 * db + 8 * g4 + 4 * hb;
      f32x4 fk = {0.f, 0.f, 0.f, 0.f}, fv = {0.f, 0.f, 0.f, 0.f};
      if (ridx >= 0) {
        for (int c = c_first; c <= c_last; ++c) {
          const int64_t slice = (int64_t)c * A.n_seqs * Hkv + head;
          const f32x4 a = *reinterpret_cast<const f32x4*>(far_dk + (slice * cap + ridx) * D + d0);
          const f32x4 b = *reinterpret_cast<const f32x4*>(far_dv + (slice * cap + ridx) * D + d0);
#pragma unroll
          for (int e = 0; e < 4; ++e) { fk[e] += a[e]; fv[e] += b[e]; }
        }
      }
      const bf16x4 v4 = *reinterpret_cast<const bf16x4*>(vrow + d0);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        dka[db][4 * g4 + e] = fmaf(dka[db][4 * g4 + e], A.scale, fk[e]);
        dva[db][4 * g4 + e] += fv[e];
        ste = fmaf(dva[db][4 * g4 + e], static_cast<float>(v4[e]), ste);
      }
    }
  ste = pair_sum(ste);
  {
    const float z = A.logits[(int64_t)h * A.total + lo + jpos];
    const bool above = key_ok && z > A.tau;
    if (key_ok && hb == 0) {
      const float r = 1.0f / (1.0f + expf(-z));
      A.dz[(int64_t)h * A.total + lo + jpos] = (ste + (above ? A.lambda[h] : 0.f)) * r * (1.0f - r);
    }
    const int c = __builtin_popcountll(__builtin_amdgcn_ballot_w64(above && hb == 0));
    if (lane == 0 && c > 0) atomicAdd(&A.counts[s * Hkv + h], c);    // integer: order does not matter
  }
  bf16_t* outs[2] = {static_cast<bf16_t*>(A.dk), static_cast<bf16_t*>(A.dv)};
#pragma unroll
  for (int which = 0; which < 2; ++which) {
    __syncthreads();
    bf16_t* orow = lds + kloc * OS + 4 * hb;
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {
        bf16x4 w4;
#pragma unroll
        for (int e = 0; e < 4; ++e) w4[e] = static_cast<bf16_t>(which == 0 ? dka[db][4 * g4 + e] : dva[db][4 * g4 + e]);
        *reinterpret_cast<bf16x4*>(orow + 32 * db + 8 * g4) = w4;
      }
    __syncthreads();
    bf16_t* obase = outs[which] + ((int64_t)(lo + j0) * Hkv + h) * D;
    const int64_t orow_stride = (int64_t)Hkv * D;
#pragma unroll
    for (int p = 0; p < BM / RPP; ++p) {
      const int row = p * RPP + k_row;
      if (j0 + row < n)
        *reinterpret_cast<u32x4*>(obase + row * orow_stride + k_piece * 8) =
            *reinterpret_cast<const u32x4*>(lds + row * OS + k_piece * 8);
    }
  }
}

// delta = <dO, O> per (query, query head), read by the dK / dV passes: eight lanes per 128-byte row.
template <int D>
__global__ void __launch_bounds__(kThreads)
train_delta_mfma_kernel(TrainArgs A) {
  constexpr int PPR = Geo<D>::PPR;
  const int64_t row = (int64_t)blockIdx.x * (kThreads / PPR) + threadIdx.x / PPR;
  const int piece = threadIdx.x % PPR;
  const int64_t rows = A.total * A.Hq;
  const int64_t rc = row < rows ? row : rows - 1;
  const bf16x8 o8 = *reinterpret_cast<const bf16x8*>(static_cast<const bf16_t*>(A.out) + rc * D + piece * 8);
  const bf16x8 d8 = *reinterpret_cast<const bf16x8*>(static_cast<const bf16_t*>(A.dout) + rc * D + piece * 8);
  float acc = 0.f;
#pragma unroll
  for (int e = 0; e < 8; ++e) acc = fmaf(static_cast<float>(d8[e]), static_cast<float>(o8[e]), acc);
#pragma unroll
  for (int off = PPR / 2; off > 0; off >>= 1) acc += __shfl_xor(acc, off, kWave);
  if (piece == 0 && row < rows) {
    const int64_t tok = row / A.Hq;
    A.delta[(row - tok * A.Hq) * A.total + tok] = acc;
  }
}

// One launch, two independent roles: the first far_blocks workgroups run the far pass of dK / dV (few, long-running:
// the candidates of early positions face almost every later query), the others compute dQ and fill the compute
// units that the far pass leaves idle.
// (D = 128 needs more than 256 registers per lane for the dK / dV role: one wave per SIMD there.)
template <int D>
__global__ void __launch_bounds__(kThreads, D == 64 ? 2 : 1)
train_dq_far_mfma_kernel(TrainArgs A, int tiles_upper, int n_work, float scale_log2e, float* far_dk, float* far_dv,
                         int far_blocks) {
  __shared__ __align__(16) bf16_t lds[2 * Geo<D>::kBuf];  // two tile buffers; the two roles lay their tiles out in them
  __shared__ __align__(16) float stat_lds[4 * BN];
  __shared__ int pos_rng[4];
  if ((int)blockIdx.x < far_blocks)
    dkv_body<D, true>(A, 0, scale_log2e, far_dk, far_dv, (int)blockIdx.x, lds, stat_lds);
  else
    dq_body<D>(A, tiles_upper, n_work, scale_log2e, (int)blockIdx.x - far_blocks, lds, reinterpret_cast<int*>(stat_lds), pos_rng);
}

template <int D>
__global__ void __launch_bounds__(kThreads, D == 64 ? 2 : 1)
train_dkv_band_mfma_kernel(TrainArgs A, int tiles_upper, float scale_log2e, float* far_dk, float* far_dv) {
  __shared__ __align__(16) bf16_t lds[2 * Geo<D>::kBufDkv];
  __shared__ __align__(16) float stat_lds[4 * BN];
  dkv_body<D, false>(A, tiles_upper, scale_log2e, far_dk, far_dv, (int)blockIdx.x, lds, stat_lds);
}

}  // namespace

// Rows are addressed with 32-bit byte offsets inside one sequence, and loaded in 16-byte pieces.
bool train_mfma_supported(const TrainArgs& A, int D) {
  if (D != 64 && D != 128) return false;
  if ((int64_t)A.max_seqlen * A.kv_st * 2 >= ((int64_t)1 << 31)) return false;
  if ((int64_t)A.max_seqlen * A.q_st * 2 >= ((int64_t)1 << 31)) return false;
  if ((int64_t)A.max_seqlen * A.Hq * D * 2 >= ((int64_t)1 << 31)) return false;
  if ((int64_t)A.budget * D * 2 >= ((int64_t)1 << 31)) return false;
  auto al16 = [](const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; };
  return al16(A.dout) && al16(A.dq) && al16(A.dk) && al16(A.dv) && al16(A.out);
}

// delta, then [far pass of dK / dV | dQ] in one launch, then the band pass of dK / dV (which adds the far pass in).
// far_dk / far_dv: fp32 scratch, [far_chunks][n_seqs * Hkv][budget][D] each (only rows below ret_count are touched).
namespace {
template <int D>
hipError_t run_mfma(const TrainArgs& A, hipStream_t stream) {
  constexpr int PPR = Geo<D>::PPR;
  const float sl2 = A.scale * 1.4426950408889634f;
  const int64_t rows = A.total * A.Hq;
  hipLaunchKernelGGL(train_delta_mfma_kernel<D>, dim3((unsigned)((rows + kThreads / PPR - 1) / (kThreads / PPR))),
                     dim3(kThreads), 0, stream, A);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const int per_head = (A.max_seqlen + BM - 1) / BM;
  int64_t far_blocks = A.budget > 0 ? (int64_t)A.n_seqs * A.Hkv * per_head * A.far_chunks : 0;
  far_blocks = (far_blocks + 7) / 8 * 8;      // keeps the dQ role's workgroup-to-XCD pattern
  const int64_t tiles_upper = (A.total + BM - 1) / BM + A.n_seqs;
  const int64_t n_work = tiles_upper * A.Hq;
  const int64_t dq_blocks = (n_work + 7) / 8 * 8;
  hipLaunchKernelGGL(train_dq_far_mfma_kernel<D>, dim3((unsigned)(far_blocks + dq_blocks)), dim3(kThreads), 0, stream, A,
                     (int)tiles_upper, (int)n_work, sl2, A.far_dk, A.far_dv, (int)far_blocks);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(train_dkv_band_mfma_kernel<D>, dim3((unsigned)((tiles_upper * A.Hkv + 7) / 8 * 8)), dim3(kThreads), 0, stream, A,
                     (int)tiles_upper, sl2, A.far_dk, A.far_dv);
  return hipGetLastError();
}
}  // namespace

hipError_t launch_train_backward_mfma(const TrainArgs& A, int D, hipStream_t stream) {
  return D == 64 ? run_mfma<64>(A, stream) : run_mfma<128>(A, stream);
}

}  // namespace ltea
