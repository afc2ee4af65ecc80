// Budgeted retention and cache fill (paper eq. 5; Section 3.1.3 "Capped capacity", "Cached prefilling").
//
// One launch.  Workgroups with blockIdx.y == 0 own one (sequence, KV head) each:
//   candidates among the out-of-window positions 0 .. n-window-1 are sinks or logits above the threshold;
//   their keys (an order-preserving integer image of the fp32 key, 0 for non-candidates) are read once and
//   stay in registers.  If more than `budget` exist, an exact radix select (up to 4 passes of 8 bits) finds
//   the budget-th largest key, and ties at that key are resolved towards lower positions by an ordered scan.
//   The same ordered scan (wave prefix sums, no atomics on results) writes the kept positions and keys
//   ascending by position, so the result is deterministic; the workgroup then gathers the kept K/V rows into
//   the compact segment.
// Workgroups with blockIdx.y >= 1 copy the last min(n, window) tokens and their logits into the ring
// (slot = position % window); that part does not depend on the selection and overlaps with it.
#include "ltea_common.h"
#include "ltea_kernels.h"

namespace ltea {
namespace {

constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / kWave;
constexpr int kItems = 4;                        // consecutive positions per thread per chunk
constexpr int kChunk = kSelThreads * kItems;     // positions per chunk
constexpr int kSub = 8;                          // sub-histograms per digit (spreads same-digit LDS atomics)
constexpr int kRingRows = 256;                   // ring rows per copy workgroup

__device__ __forceinline__ float key_of_order_key(uint32_t u) {
  return __uint_as_float((u & 0x80000000u) ? (u ^ 0x80000000u) : ~u);
}

// Exclusive prefix sum of `val` over the block (thread order); `total` receives the block sum.
// `scratch` holds kSelWaves+1 ints of LDS. Contains two barriers.
__device__ __forceinline__ int block_exclusive_scan(int val, int* scratch, int& total) {
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  int inc = val;
#pragma unroll
  for (int off = 1; off < kWave; off <<= 1) {
    int t = __shfl_up(inc, off, kWave);
    if (lane >= off) inc += t;
  }
  __syncthreads();  // protect scratch from the previous use
  if (lane == kWave - 1) scratch[wave] = inc;
  __syncthreads();
  int before = 0, all = 0;
#pragma unroll
  for (int w = 0; w < kSelWaves; ++w) {
    int t = scratch[w];
    if (w < wave) before += t;
    all += t;
  }
  total = all;
  return before + inc - val;
}

struct RetainArgs {
  const float* logits; int64_t total; const int32_t* cu; int Hkv, window, budget, sink; float tau; int rho;
  const char* k; const char* v; int64_t tok_bytes, head_bytes; int row_bytes;   // K/V views in bytes
  char* k_win; char* v_win; float* win_score; char* k_ret; char* v_ret;
  float* ret_score; int32_t* ret_pos; int32_t* ret_count; int32_t* n_seen; int32_t* n_scored;
};

// Copies one K row and one V row of row_bytes (a multiple of 16) in 16-byte pieces; piece index `pc`.
__device__ __forceinline__ void copy_piece(const RetainArgs& a, int64_t src_off, char* dk, char* dv, int pc) {
  reinterpret_cast<u32x4*>(dk)[pc] = reinterpret_cast<const u32x4*>(a.k + src_off)[pc];
  reinterpret_cast<u32x4*>(dv)[pc] = reinterpret_cast<const u32x4*>(a.v + src_off)[pc];
}

// CH > 0: the (sequence, head)'s out-of-window keys fit CH chunks and are held in registers;
// CH == 0: any length, keys are re-read from memory in every pass.
template <int CH>
__global__ void __launch_bounds__(kSelThreads)
retain_kernel(const RetainArgs a) {
  __shared__ int scan_scratch[kSelWaves + 1];
  __shared__ __align__(16) int hist[256 * kSub];
  __shared__ int sel_digit, sel_need, sel_total, sel_exact;

  const int b = blockIdx.x / a.Hkv, h = blockIdx.x - b * a.Hkv;
  const int tid = threadIdx.x, lane = tid & (kWave - 1);
  const int64_t lo = a.cu[b];
  const int n = (int)(a.cu[b + 1] - lo);
  const int64_t head = (int64_t)b * a.Hkv + h;
  const float* z = a.logits + (int64_t)h * a.total + lo;
  const int pieces = a.row_bytes / 16;

  if (blockIdx.y > 0) {
    // ---- ring rows: slot -> the position it holds after n tokens ----
    const int rows_per_pass = kSelThreads / pieces;
    const int sub = tid / pieces, pc = tid - sub * pieces;
    const int row_end = min((int)blockIdx.y * kRingRows, a.window);
    for (int slot = ((int)blockIdx.y - 1) * kRingRows + sub; slot < row_end; slot += rows_per_pass) {
      int p;
      if (n >= a.window) {
        const int first = n - a.window;   // oldest position in the window
        p = first + (slot - first % a.window + a.window) % a.window;
      } else {
        p = slot < n ? slot : -1;
      }
      if (p < 0) continue;
      if (pc == 0) a.win_score[head * a.window + slot] = z[p];
      copy_piece(a, (lo + p) * a.tok_bytes + h * a.head_bytes, a.k_win + (head * a.window + slot) * a.row_bytes,
                 a.v_win + (head * a.window + slot) * a.row_bytes, pc);
    }
    return;
  }

  const int n_out = n > a.window ? n - a.window : 0;
  if (h == 0 && tid == 0) {
    a.n_seen[b] = n;
    a.n_scored[b] = n > a.rho ? n - a.rho : 0;
  }
  if (a.budget == 0 || n_out == 0) {
    if (tid == 0) a.ret_count[head] = 0;
    return;
  }

  // ---- keys: 0 = not a candidate (every candidate's order key is positive) ----
  auto fetch = [&](int j) -> uint32_t {
    if (j >= n_out) return 0u;
    const float zj = z[j];
    return ((j < a.sink) || (zj > a.tau)) ? order_key(select_key(zj, j, a.sink)) : 0u;
  };
  constexpr int kHeld = CH > 0 ? CH : 1;
  uint32_t held[kHeld][kItems];
  if constexpr (CH > 0) {
    // a thread's four logits of a chunk are consecutive: one 16-byte load where the head's row allows it
    static_assert(kItems == 4, "one float4 per thread and chunk");
    const bool quads = (reinterpret_cast<uintptr_t>(z) & 15u) == 0;
    auto key_of = [&](float zj, int j) -> uint32_t {
      return ((j < a.sink) || (zj > a.tau)) ? order_key(select_key(zj, j, a.sink)) : 0u;
    };
#pragma unroll
    for (int c = 0; c < CH; ++c) {
      const int j0 = c * kChunk + tid * kItems;
      if (quads && j0 + kItems <= n_out) {
        const float4 z4 = *reinterpret_cast<const float4*>(z + j0);
        held[c][0] = key_of(z4.x, j0); held[c][1] = key_of(z4.y, j0 + 1);
        held[c][2] = key_of(z4.z, j0 + 2); held[c][3] = key_of(z4.w, j0 + 3);
      } else {
#pragma unroll
        for (int e = 0; e < kItems; ++e) held[c][e] = fetch(j0 + e);
      }
    }
  }
  const int n_chunks = (n_out + kChunk - 1) / kChunk;
  // A sequence longer than the caller's max_seqlen (which picked CH) does not fit the held registers: its keys are
  // re-read from memory in every pass instead (a workgroup-uniform choice), so the result stays exact.
  const bool use_held = CH > 0 && n_chunks <= CH;
  auto chunk_keys = [&](int c, uint32_t (&u)[kItems]) {
    if (use_held) {
#pragma unroll
      for (int cc = 0; cc < kHeld; ++cc)
        if (cc == c) {
#pragma unroll
          for (int e = 0; e < kItems; ++e) u[e] = held[cc][e];
        }
    } else {
#pragma unroll
      for (int e = 0; e < kItems; ++e) u[e] = fetch(c * kChunk + tid * kItems + e);
    }
  };

  // ---- exact budget-th largest key (only when the cap binds); the first pass also counts the candidates ----
  uint32_t thr = 0;      // keep keys strictly above thr ...
  int need_eq = 0;       // ... plus the first need_eq (by position) equal to thr
  {
    uint32_t prefix = 0;
    int need = a.budget;
    for (int pass = 0; pass < 4; ++pass) {
      const int shift = 24 - 8 * pass;
      hist[tid] = 0;
      hist[tid + kSelThreads] = 0;
      __syncthreads();
#pragma unroll 1
      for (int c = 0; c < n_chunks; ++c) {
        uint32_t u[kItems];
        chunk_keys(c, u);
#pragma unroll
        for (int e = 0; e < kItems; ++e) {
          const bool match = u[e] != 0u && ((pass == 0) || ((u[e] >> (shift + 8)) == prefix));
          if (match) atomicAdd(&hist[((u[e] >> shift) & 255u) * kSub + (lane & (kSub - 1))], 1);
        }
      }
      __syncthreads();
      if (tid < kWave) {
        // lane l owns digits 255-4l .. 252-4l, so lane order is descending digit order
        int cnt[4], mine = 0;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int d = 255 - 4 * lane - i;
          const int4 x = *reinterpret_cast<const int4*>(&hist[d * kSub]);
          const int4 y = *reinterpret_cast<const int4*>(&hist[d * kSub + 4]);
          cnt[i] = x.x + x.y + x.z + x.w + y.x + y.y + y.z + y.w;
          mine += cnt[i];
        }
        int inc = mine;
#pragma unroll
        for (int off = 1; off < kWave; off <<= 1) {
          const int t = __shfl_up(inc, off, kWave);
          if (lane >= off) inc += t;
        }
        int running = inc - mine;   // elements with a larger digit than this lane's first
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          if (running < need && need <= running + cnt[i]) {
            sel_digit = 255 - 4 * lane - i;
            sel_need = need - running;
            sel_exact = need == running + cnt[i];   // the whole bucket is kept: the lower digits decide nothing
          }
          running += cnt[i];
        }
        if (lane == kWave - 1) sel_total = inc;
      }
      __syncthreads();
      if (pass == 0 && sel_total <= a.budget) break;   // the cap does not bind: keep every candidate
      prefix = (prefix << 8) | (uint32_t)sel_digit;
      need = sel_need;
      if (pass == 3) { thr = prefix; need_eq = need; }
      else if (sel_exact && (prefix << shift) != 0u) { thr = (prefix << shift) - 1u; break; }   // keep keys >= prefix << shift
      __syncthreads();   // hist and sel_* are rewritten by the next pass
    }
  }

  // ---- ordered compaction: ascending positions ----
  int kept_before = 0, eq_before = 0;
#pragma unroll 1
  for (int c = 0; c < n_chunks; ++c) {
    const int j0 = c * kChunk + tid * kItems;
    uint32_t u[kItems];
    chunk_keys(c, u);
    int n_eq = 0;
#pragma unroll
    for (int e = 0; e < kItems; ++e) n_eq += (need_eq > 0 && u[e] == thr);
    int eq_rank = 0, eq_total = 0;
    if (need_eq > 0) eq_rank = eq_before + block_exclusive_scan(n_eq, scan_scratch, eq_total);
    bool keep[kItems];
    int n_keep = 0;
#pragma unroll
    for (int e = 0; e < kItems; ++e) {
      bool kp = false;
      if (u[e] > thr) kp = true;
      else if (need_eq > 0 && u[e] == thr) { kp = eq_rank < need_eq; ++eq_rank; }
      keep[e] = kp;
      n_keep += kp;
    }
    int keep_total;
    int off = kept_before + block_exclusive_scan(n_keep, scan_scratch, keep_total);
#pragma unroll
    for (int e = 0; e < kItems; ++e) {
      if (keep[e]) {
        a.ret_pos[head * a.budget + off] = j0 + e;
        a.ret_score[head * a.budget + off] = key_of_order_key(u[e]);
        ++off;
      }
    }
    kept_before += keep_total;
    eq_before += eq_total;
  }
  if (tid == 0) a.ret_count[head] = kept_before;

  // ---- gather the kept rows (positions written above by this workgroup) ----
  __threadfence_block();
  __syncthreads();
  // four pieces per thread in flight: positions first, then all the row loads, then the stores
  constexpr int kGather = 4;
  const int n_pieces = kept_before * pieces;
  for (int i0 = tid; i0 < n_pieces; i0 += kGather * kSelThreads) {
    int r[kGather], pc[kGather], p[kGather];
#pragma unroll
    for (int u = 0; u < kGather; ++u) {
      const int i = i0 + u * kSelThreads;
      const int ic = i < n_pieces ? i : i0;          // past the end: this thread's first piece once more, not stored
      r[u] = ic / pieces;
      pc[u] = ic - r[u] * pieces;
      p[u] = a.ret_pos[head * a.budget + r[u]];
    }
    u32x4 xk[kGather], xv[kGather];
#pragma unroll
    for (int u = 0; u < kGather; ++u) {
      const int64_t src = (lo + p[u]) * a.tok_bytes + h * a.head_bytes;
      xk[u] = reinterpret_cast<const u32x4*>(a.k + src)[pc[u]];
      xv[u] = reinterpret_cast<const u32x4*>(a.v + src)[pc[u]];
    }
#pragma unroll
    for (int u = 0; u < kGather; ++u) {
      if (i0 + u * kSelThreads < n_pieces) {
        reinterpret_cast<u32x4*>(a.k_ret + (head * a.budget + r[u]) * a.row_bytes)[pc[u]] = xk[u];
        reinterpret_cast<u32x4*>(a.v_ret + (head * a.budget + r[u]) * a.row_bytes)[pc[u]] = xv[u];
      }
    }
  }
}

}  // namespace

hipError_t launch_retain(const ltea_cfg& cfg, const float* logits, const void* k, const void* v, int64_t stride_tok,
                         int64_t stride_head, const SeqView& sv, int rho, const ltea_cache& c, hipStream_t stream) {
  if (sv.n_seqs == 0) return hipSuccess;
  const int64_t esz = cfg.dtype == LTEA_F32 ? 4 : 2;
  RetainArgs a;
  a.logits = logits; a.total = sv.total_tokens; a.cu = sv.cu_seqlens; a.Hkv = cfg.Hkv; a.window = cfg.window;
  a.budget = cfg.budget; a.sink = cfg.sink; a.tau = cfg.tau_logit; a.rho = rho;
  a.k = static_cast<const char*>(k); a.v = static_cast<const char*>(v);
  a.tok_bytes = stride_tok * esz; a.head_bytes = stride_head * esz; a.row_bytes = (int)(cfg.D * esz);
  a.k_win = static_cast<char*>(c.k_win); a.v_win = static_cast<char*>(c.v_win); a.win_score = c.win_score;
  a.k_ret = static_cast<char*>(c.k_ret); a.v_ret = static_cast<char*>(c.v_ret);
  a.ret_score = c.ret_score; a.ret_pos = c.ret_pos; a.ret_count = c.ret_count; a.n_seen = c.n_seen;
  a.n_scored = c.n_scored;
  const unsigned heads = (unsigned)sv.n_seqs * (unsigned)cfg.Hkv;
  const dim3 grid(heads, 1u + (unsigned)((cfg.window + kRingRows - 1) / kRingRows));
  const int64_t n_out_max = sv.max_seqlen > cfg.window ? sv.max_seqlen - cfg.window : 0;
  if (n_out_max <= 1 * kChunk) hipLaunchKernelGGL(retain_kernel<1>, grid, dim3(kSelThreads), 0, stream, a);
  else if (n_out_max <= 2 * kChunk) hipLaunchKernelGGL(retain_kernel<2>, grid, dim3(kSelThreads), 0, stream, a);
  else if (n_out_max <= 4 * kChunk) hipLaunchKernelGGL(retain_kernel<4>, grid, dim3(kSelThreads), 0, stream, a);
  else if (n_out_max <= 8 * kChunk) hipLaunchKernelGGL(retain_kernel<8>, grid, dim3(kSelThreads), 0, stream, a);
  else hipLaunchKernelGGL(retain_kernel<0>, grid, dim3(kSelThreads), 0, stream, a);
  return hipGetLastError();
}

}  // namespace ltea
