// Budgeted retention and cache fill (paper eq. 5; Section 3.1.3 "Capped capacity", "Cached prefilling").
//
// Kernel 1 (retain_select_kernel), one workgroup per (sequence, KV head):
//   candidates among the out-of-window positions 0 .. n-window-1 are sinks or logits above the threshold;
//   if more than `budget` exist, an exact radix select (4 passes of 8 bits over an order-preserving
//   integer image of the fp32 key) finds the budget-th largest key, and ties at that key are resolved
//   towards lower positions by an ordered scan.  The same ordered scan (wave prefix sums, no atomics on
//   results) writes the kept positions and keys ascending by position, so the result is deterministic.
// Kernel 2 (cache_fill_kernel): gathers the kept K/V rows into the compact segment and copies the last
//   min(n, window) tokens and their logits into the ring (slot = position % window).
#include "ltea_common.h"
#include "ltea_kernels.h"

namespace ltea {
namespace {

constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / kWave;
constexpr int kItems = 4;  // consecutive positions per thread per chunk

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

__global__ void __launch_bounds__(kSelThreads)
retain_select_kernel(const float* __restrict__ logits, int64_t total, const int32_t* __restrict__ cu, int Hkv,
                     int window, int budget, int sink, float tau, int rho, float* __restrict__ ret_score,
                     int32_t* __restrict__ ret_pos, int32_t* __restrict__ ret_count, int32_t* __restrict__ n_seen,
                     int32_t* __restrict__ n_scored) {
  __shared__ int scan_scratch[kSelWaves + 1];
  __shared__ int hist[256];
  __shared__ int sel_digit, sel_need;

  const int b = blockIdx.x / Hkv, h = blockIdx.x - b * Hkv;
  const int tid = threadIdx.x;
  const int64_t lo = cu[b];
  const int n = (int)(cu[b + 1] - lo);
  const int n_out = n > window ? n - window : 0;
  const float* z = logits + (int64_t)h * total + lo;
  if (h == 0 && tid == 0) {
    n_seen[b] = n;
    n_scored[b] = n > rho ? n - rho : 0;
  }
  const int64_t head = (int64_t)b * Hkv + h;
  if (budget == 0 || n_out == 0) {
    if (tid == 0) ret_count[head] = 0;
    return;
  }

  // ---- count candidates ----
  int mine = 0;
  for (int j = tid; j < n_out; j += kSelThreads) {
    const float zj = z[j];
    mine += (j < sink) || (zj > tau);
  }
  int n_cand;
  block_exclusive_scan(mine, scan_scratch, n_cand);

  // ---- exact budget-th largest key (only when the cap binds) ----
  uint32_t thr = 0;      // keep keys strictly above thr ...
  int need_eq = 0;       // ... plus the first need_eq (by position) equal to thr
  if (n_cand > budget) {
    uint32_t prefix = 0;
    int need = budget;
    for (int pass = 0; pass < 4; ++pass) {
      const int shift = 24 - 8 * pass;
      if (tid < 256) hist[tid] = 0;
      __syncthreads();
      for (int j = tid; j < n_out; j += kSelThreads) {
        const float zj = z[j];
        if ((j < sink) || (zj > tau)) {
          const uint32_t u = order_key(select_key(zj, j, sink));
          const bool match = (pass == 0) || ((u >> (shift + 8)) == prefix);
          if (match) atomicAdd(&hist[(u >> shift) & 255u], 1);
        }
      }
      __syncthreads();
      // threads 0..255 walk the digits from 255 down: thread i owns digit 255-i.
      int cnt = (tid < 256) ? hist[255 - tid] : 0;
      int tot;
      int before = block_exclusive_scan(cnt, scan_scratch, tot);  // elements with a larger digit
      if (tid < 256 && before < need && need <= before + cnt) {
        sel_digit = 255 - tid;
        sel_need = need - before;
      }
      __syncthreads();
      prefix = (prefix << 8) | (uint32_t)sel_digit;
      need = sel_need;
      __syncthreads();
    }
    thr = prefix;
    need_eq = need;
  }

  // ---- ordered compaction: ascending positions ----
  int kept_before = 0, eq_before = 0;
  const int chunk = kSelThreads * kItems;
  for (int base = 0; base < n_out; base += chunk) {
    const int j0 = base + tid * kItems;
    uint32_t u[kItems];
    float key[kItems];
    bool cand[kItems];
    int n_eq = 0;
#pragma unroll
    for (int e = 0; e < kItems; ++e) {
      const int j = j0 + e;
      cand[e] = false;
      u[e] = 0;
      key[e] = 0.f;
      if (j < n_out) {
        const float zj = z[j];
        cand[e] = (j < sink) || (zj > tau);
        key[e] = select_key(zj, j, sink);
        u[e] = order_key(key[e]);
      }
      n_eq += (cand[e] && need_eq > 0 && u[e] == thr);
    }
    int eq_rank = 0, eq_total = 0;
    if (need_eq > 0) eq_rank = eq_before + block_exclusive_scan(n_eq, scan_scratch, eq_total);
    bool keep[kItems];
    int n_keep = 0;
#pragma unroll
    for (int e = 0; e < kItems; ++e) {
      bool kp = false;
      if (cand[e]) {
        if (u[e] > thr) kp = true;
        else if (need_eq > 0 && u[e] == thr) { kp = eq_rank < need_eq; ++eq_rank; }
      }
      keep[e] = kp;
      n_keep += kp;
    }
    int keep_total;
    int off = kept_before + block_exclusive_scan(n_keep, scan_scratch, keep_total);
#pragma unroll
    for (int e = 0; e < kItems; ++e) {
      if (keep[e]) {
        ret_pos[head * budget + off] = j0 + e;
        ret_score[head * budget + off] = key[e];
        ++off;
      }
    }
    kept_before += keep_total;
    eq_before += eq_total;
  }
  if (tid == 0) ret_count[head] = kept_before;
}

// Rows 0..budget-1 of the grid's row space are compact slots, rows budget..budget+window-1 ring slots.
// Each row is copied in 16-byte pieces (D*sizeof(T) is a multiple of 16 and rows are 16-byte aligned).
template <typename T>
__global__ void __launch_bounds__(256)
cache_fill_kernel(const T* __restrict__ k, const T* __restrict__ v, int64_t stride_tok, int64_t stride_head, int D,
                  const float* __restrict__ logits, int64_t total, const int32_t* __restrict__ cu, int Hkv,
                  int window, int budget, T* __restrict__ k_win, T* __restrict__ v_win,
                  float* __restrict__ win_score, T* __restrict__ k_ret, T* __restrict__ v_ret,
                  const int32_t* __restrict__ ret_pos, const int32_t* __restrict__ ret_count, int rows_per_block) {
  const int b = blockIdx.x / Hkv, h = blockIdx.x - b * Hkv;
  const int64_t head = (int64_t)b * Hkv + h;
  const int64_t lo = cu[b];
  const int n = (int)(cu[b + 1] - lo);
  const int pieces = D * (int)sizeof(T) / 16;  // 16-byte pieces per row
  const int rows_per_pass = 256 / pieces;
  const int sub = threadIdx.x / pieces, piece = threadIdx.x - sub * pieces;
  const int cnt = ret_count[head];
  const int row_end = min((int)(blockIdx.y + 1) * rows_per_block, budget + window);
  for (int r = blockIdx.y * rows_per_block + sub; r < row_end; r += rows_per_pass) {
    int p;        // source position inside the sequence, or -1
    T *dk, *dv;
    if (r < budget) {
      p = r < cnt ? ret_pos[head * budget + r] : -1;
      dk = k_ret + (head * budget + r) * D;
      dv = v_ret + (head * budget + r) * D;
    } else {
      const int slot = r - budget;
      if (n >= window) {
        const int first = n - window;                    // oldest position in the window
        int d = (slot - first % window + window) % window;
        p = first + d;
      } else {
        p = slot < n ? slot : -1;
      }
      dk = k_win + (head * window + slot) * D;
      dv = v_win + (head * window + slot) * D;
      if (p >= 0 && piece == 0) win_score[head * window + slot] = logits[(int64_t)h * total + lo + p];
    }
    if (p < 0) continue;
    const T* sk = k + (lo + p) * stride_tok + (int64_t)h * stride_head;
    const T* sv = v + (lo + p) * stride_tok + (int64_t)h * stride_head;
    reinterpret_cast<u32x4*>(dk)[piece] = reinterpret_cast<const u32x4*>(sk)[piece];
    reinterpret_cast<u32x4*>(dv)[piece] = reinterpret_cast<const u32x4*>(sv)[piece];
  }
}

}  // namespace

hipError_t launch_retain(const ltea_cfg& cfg, const float* logits, const void* k, const void* v, int64_t stride_tok,
                         int64_t stride_head, const SeqView& sv, int rho, const ltea_cache& c, hipStream_t stream) {
  if (sv.n_seqs == 0) return hipSuccess;
  const unsigned heads = (unsigned)sv.n_seqs * (unsigned)cfg.Hkv;
  hipLaunchKernelGGL(retain_select_kernel, dim3(heads), dim3(kSelThreads), 0, stream, logits, sv.total_tokens,
                     sv.cu_seqlens, cfg.Hkv, cfg.window, cfg.budget, cfg.sink, cfg.tau_logit, rho, c.ret_score,
                     c.ret_pos, c.ret_count, c.n_seen, c.n_scored);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const int rows = cfg.budget + cfg.window;
  const int rows_per_block = 128;
  dim3 grid(heads, (unsigned)((rows + rows_per_block - 1) / rows_per_block));
  if (cfg.dtype == LTEA_F32) {
    hipLaunchKernelGGL(cache_fill_kernel<float>, grid, dim3(256), 0, stream, static_cast<const float*>(k),
                       static_cast<const float*>(v), stride_tok, stride_head, cfg.D, logits, sv.total_tokens,
                       sv.cu_seqlens, cfg.Hkv, cfg.window, cfg.budget, static_cast<float*>(c.k_win),
                       static_cast<float*>(c.v_win), c.win_score, static_cast<float*>(c.k_ret),
                       static_cast<float*>(c.v_ret), c.ret_pos, c.ret_count, rows_per_block);
  } else {
    hipLaunchKernelGGL(cache_fill_kernel<bf16_t>, grid, dim3(256), 0, stream, static_cast<const bf16_t*>(k),
                       static_cast<const bf16_t*>(v), stride_tok, stride_head, cfg.D, logits, sv.total_tokens,
                       sv.cu_seqlens, cfg.Hkv, cfg.window, cfg.budget, static_cast<bf16_t*>(c.k_win),
                       static_cast<bf16_t*>(c.v_win), c.win_score, static_cast<bf16_t*>(c.k_ret),
                       static_cast<bf16_t*>(c.v_ret), c.ret_pos, c.ret_count, rows_per_block);
  }
  return hipGetLastError();
}

}  // namespace ltea
