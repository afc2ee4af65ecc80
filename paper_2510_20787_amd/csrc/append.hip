// Continuation of a prefill onto an existing cache state (paper Section 3.1.3: the state after N tokens is the
// ring of the last w tokens plus the capped out-of-window segment; tokens dropped earlier are gone for good).
//
// Appending M new tokens to a sequence must give the rows and the final state of a one-shot prefill over all
// N + M tokens.  That holds because the kept set is nested: a token that is not among the top-b candidates of a
// prefix cannot be among the top-b of a longer one, so top-b over (old kept set + tokens leaving the window now)
// equals top-b over everything.
//
// The work is put in the shape the prefill kernels already handle.  Per sequence an "extended sequence" is laid out
// in the workspace:   [ pad | old kept entries ascending by position | ring tokens in position order | new tokens ]
// with the prefix (pad + kept entries) given the same length F for every head of the sequence, F >= budget chosen
// such that extended index and true position agree modulo the window (so that the ring slot of a token, position %
// window, can be computed from either).  Then
//   1. the scoring kernel runs over the extended sequence; logits of ring tokens that were already final are taken
//      from the cache instead (their left context may be outside the ring), prefix entries get their stored keys,
//      pad entries NaN (never candidates; their K/V rows are zero, and the scoring is told that a sequence which
//      started inside the ring begins after them: cu_score);
//   2. the retention kernel runs over the extended sequence (candidates, top-b, gather, ring fill) unchanged;
//   3. kept positions are translated back from extended indices to true positions, counters are set;
//   4. the attention kernel runs with the ring + new part of the extended sequence as keys and the new tokens as
//      queries (kept positions expressed in that local frame; old kept entries get negative positions and are visible
//      to every new query, as they should be).
// Rotary models cache the keys after the rotation while the CNN scores them as they were before it.  For them the
// extended sequence gets a second key buffer that only the scoring kernel reads: ring rows rotated back with the
// model's sinusoids (as in the batched scoring of the decode ring), new rows taken from the caller's unrotated keys or
// rotated back as well.
#include "ltea_common.h"
#include "ltea_kernels.h"
#include "rope_dev.h"

namespace ltea {
namespace {

struct AppendPlan {        // device arrays in the workspace, one entry per sequence unless noted
  int32_t* n_old;          // tokens in the cache before the call
  int32_t* w_old;          // min(n_old, window): ring tokens
  int32_t* prefix;         // F
  int32_t* cu_ext;         // [n_seqs + 1] packing of the extended sequences
  int32_t* cu_score;       // [n_seqs + 1] the same packing as the scoring kernels must see it (see the plan kernel)
  int32_t* kv_start;       // first row of the ring + new part in the extended buffers
  int32_t* kv_len;         // w_old + new tokens
  int32_t* sorted_pos;     // [n_seqs][Hkv][budget] old kept positions ascending
  int32_t* sorted_slot;    // [n_seqs][Hkv][budget] compact slot of the entry with that rank
  int32_t* local_pos;      // [n_seqs][Hkv][budget] kept positions in the ring + new frame (for the attention kernel)
};

__device__ __forceinline__ void plan_body(const AppendPlan& P, const int32_t* __restrict__ cu_new,
                                          const int32_t* __restrict__ n_seen, int n_seqs, int window, int budget) {
  // one workgroup: sequential prefix sum over the sequences (a handful to a few thousand)
  __shared__ int carry;
  if (threadIdx.x == 0) carry = 0;
  __syncthreads();
  for (int s0 = 0; s0 < n_seqs; s0 += 256) {
    const int s = s0 + threadIdx.x;
    int ext = 0, N = 0, wo = 0, F = 0, M = 0;
    if (s < n_seqs) {
      N = n_seen[s];
      wo = N < window ? N : window;
      M = cu_new[s + 1] - cu_new[s];
      const int want = (N - wo) % window;             // true position of the first ring token, modulo the window
      F = budget + ((want - budget) % window + window) % window;   // smallest F >= budget with F == want (mod window)
      ext = F + wo + M;
    }
    // inclusive scan over the 256 threads (4 waves)
    __shared__ int wave_tot[4];
    int inc = ext;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
      const int t = __shfl_up(inc, off, kWave);
      if (lane >= off) inc += t;
    }
    if (lane == kWave - 1) wave_tot[wave] = inc;
    __syncthreads();
    int before = carry;
    for (int w = 0; w < wave; ++w) before += wave_tot[w];
    if (s < n_seqs) {
      const int start = before + inc - ext;
      P.n_old[s] = N; P.w_old[s] = wo; P.prefix[s] = F;
      P.cu_ext[s] = start;
      // A sequence whose ring still begins at position 0 has only pad rows in its prefix.  For the scoring they
      // must not exist at all (a conv stack pads with zeros at every layer, and a zero input row does not give a
      // zero activation), so the scoring sees this sequence begin after its pad; the pad then trails the previous
      // sequence, where it can only reach logits that are provisional anyway.
      P.cu_score[s] = start + (N <= window ? F : 0);
      P.kv_start[s] = start + F;
      P.kv_len[s] = wo + M;
      if (s == n_seqs - 1) { P.cu_ext[n_seqs] = start + ext; P.cu_score[n_seqs] = start + ext; }
    }
    __syncthreads();
    if (threadIdx.x == 255) carry = before + inc;
    __syncthreads();
  }
}

// Rank of every old kept entry by position (positions are distinct): O(count^2 / threads), count <= budget.
__device__ __forceinline__ void rank_body(const AppendPlan& P, int64_t head, const int32_t* __restrict__ ret_pos,
                                          const int32_t* __restrict__ ret_count, int budget,
                                          int32_t* __restrict__ old_count) {
  const int cnt = budget > 0 ? ret_count[head] : 0;
  if (threadIdx.x == 0) old_count[head] = cnt;   // the retention stage overwrites ret_count; the translation stage needs this
  const int32_t* pos = ret_pos + head * budget;
  for (int i = threadIdx.x; i < cnt; i += 256) {
    const int p = pos[i];
    int rank = 0;
    for (int j = 0; j < cnt; ++j) rank += pos[j] < p;
    P.sorted_pos[head * budget + rank] = p;
    P.sorted_slot[head * budget + rank] = i;
  }
}

// One launch for both preparations (they do not depend on each other): workgroup 0 plans, workgroup 1 + head ranks.
__global__ void __launch_bounds__(256)
append_plan_rank_kernel(AppendPlan P, const int32_t* __restrict__ cu_new, const int32_t* __restrict__ n_seen, int n_seqs,
                        int window, int budget, const int32_t* __restrict__ ret_pos,
                        const int32_t* __restrict__ ret_count, int32_t* __restrict__ old_count) {
  if (blockIdx.x == 0) plan_body(P, cu_new, n_seen, n_seqs, window, budget);
  else rank_body(P, (int64_t)blockIdx.x - 1, ret_pos, ret_count, budget, old_count);
}

struct BuildArgs {
  const char* k_new; const char* v_new; int64_t tok_bytes, head_bytes;   // new tokens [T][Hkv][D] view, in bytes
  const char* kf_new;                // the new tokens' keys as the CNN wants them (same view), or null
  const int32_t* cu_new;
  const char* k_win; const char* v_win; const char* k_ret; const char* v_ret; const int32_t* ret_count;
  char* k_ext; char* v_ext;          // [total_ext][Hkv][D] contiguous
  char* kf_ext;                      // scoring keys of the extended rows, or null when they are the cached keys
  RopeDev rope;                      // cos == null: no rotation to undo
  int32_t* status;
  int Hkv, window, budget, row_bytes;
};

// Extended K/V rows of one (sequence, head): blockIdx.y walks chunks of 128 extended rows.
template <typename T>
__global__ void __launch_bounds__(256)
append_build_kernel(AppendPlan P, BuildArgs a) {
  constexpr int EPP = Elems<T>::N;
  const int b = blockIdx.x / a.Hkv, h = blockIdx.x - b * a.Hkv;
  const int64_t head = (int64_t)b * a.Hkv + h;
  const int N = P.n_old[b], wo = P.w_old[b], F = P.prefix[b];
  const int e0 = P.cu_ext[b], len = P.cu_ext[b + 1] - e0;
  const int cnt = a.budget > 0 ? a.ret_count[head] : 0, pad = F - cnt;
  const int pieces = a.row_bytes / 16, rows_per_pass = 256 / pieces;
  const int sub = threadIdx.x / pieces, pc = threadIdx.x - sub * pieces;
  const int row_end = min((int)(blockIdx.y + 1) * 128, len);
  const int64_t new0 = a.cu_new[b];
  bool out_of_tables = false;
  for (int e = blockIdx.y * 128 + sub; e < row_end; e += rows_per_pass) {
    const char* sk = nullptr;
    const char* sv = nullptr;
    const char* sf = nullptr;   // a row of ready-made scoring keys
    int p_rot = -1;             // position whose rotation has to be undone for the scoring keys
    if (e < pad) {
      // zero rows
    } else if (e < F) {
      // an old kept entry: only its stored key takes part in the selection, its rows never reach a logit that is used
      const int slot = P.sorted_slot[head * a.budget + (e - pad)];
      sk = a.k_ret + (head * a.budget + slot) * a.row_bytes;
      sv = a.v_ret + (head * a.budget + slot) * a.row_bytes;
    } else if (e < F + wo) {
      const int p = N - wo + (e - F);                       // true position of this ring token
      const int slot = p % a.window;
      sk = a.k_win + (head * a.window + slot) * a.row_bytes;
      sv = a.v_win + (head * a.window + slot) * a.row_bytes;
      p_rot = p;
    } else {
      const int64_t t = new0 + (e - F - wo);
      sk = a.k_new + t * a.tok_bytes + h * a.head_bytes;
      sv = a.v_new + t * a.tok_bytes + h * a.head_bytes;
      if (a.kf_new != nullptr) sf = a.kf_new + t * a.tok_bytes + h * a.head_bytes;
      else p_rot = N + (e - F - wo);
    }
    u32x4 xk = {0u, 0u, 0u, 0u}, xv = {0u, 0u, 0u, 0u};
    if (sk != nullptr) {
      xk = reinterpret_cast<const u32x4*>(sk)[pc];
      xv = reinterpret_cast<const u32x4*>(sv)[pc];
    }
    const int64_t dst = ((int64_t)(e0 + e) * a.Hkv + h) * a.row_bytes;
    reinterpret_cast<u32x4*>(a.k_ext + dst)[pc] = xk;
    reinterpret_cast<u32x4*>(a.v_ext + dst)[pc] = xv;
    if (a.kf_ext != nullptr) {
      u32x4 xf = xk;
      if (sf != nullptr) {
        xf = reinterpret_cast<const u32x4*>(sf)[pc];
      } else if (p_rot >= 0 && a.rope.cos != nullptr && pc * EPP < a.rope.rot_dim) {
        if (p_rot >= a.rope.n_pos) out_of_tables = true;
        else xf = unrotate_piece<T>(a.rope, p_rot, pc * EPP, xk, reinterpret_cast<const T*>(sk));
      }
      reinterpret_cast<u32x4*>(a.kf_ext + dst)[pc] = xf;
    }
  }
  if (out_of_tables && a.status != nullptr) atomicOr(a.status, LTEA_ROPE_RANGE);
}

// Selection keys over the extended sequence, written over the logits the scoring kernel produced.
__global__ void __launch_bounds__(256)
append_keys_kernel(AppendPlan P, float* __restrict__ ext_logits, int64_t total_ext, const float* __restrict__ win_score,
                   const float* __restrict__ ret_score, const int32_t* __restrict__ ret_count, int Hkv, int window,
                   int budget, int sink, int rho) {
  const int b = blockIdx.x / Hkv, h = blockIdx.x - b * Hkv;
  const int64_t head = (int64_t)b * Hkv + h;
  const int N = P.n_old[b], wo = P.w_old[b], F = P.prefix[b];
  const int e0 = P.cu_ext[b], len = P.cu_ext[b + 1] - e0;
  const int cnt = budget > 0 ? ret_count[head] : 0, pad = F - cnt;
  float* z = ext_logits + (int64_t)h * total_ext + e0;
  for (int e = blockIdx.y * 1024 + threadIdx.x; e < min((int)(blockIdx.y + 1) * 1024, len); e += 256) {
    if (e < pad) {
      z[e] = __uint_as_float(0x7FC00000u);                   // NaN: never a candidate
    } else if (e < F) {
      z[e] = ret_score[head * budget + P.sorted_slot[head * budget + (e - pad)]];
    } else {
      const int p = N - wo + (e - F);                        // true position
      // sinks always stay; only positions that leave the window now need the key (those that remain in the ring keep
      // their logit, which is what the ring stores)
      if (p < sink && e < len - window) z[e] = __uint_as_float(0x7F800000u);
      else if (p < N - rho) z[e] = win_score[head * window + p % window];   // final before this call
      // else: the logit just computed (final if its right context is complete, provisional otherwise)
    }
  }
}

// Kept positions back to true positions (and to the ring + new frame for the attention kernel); counters.
__global__ void __launch_bounds__(256)
append_fixup_kernel(AppendPlan P, const int32_t* __restrict__ cu_new, int32_t* __restrict__ ret_pos,
                    const int32_t* __restrict__ ret_count, const int32_t* __restrict__ old_count,
                    int32_t* __restrict__ n_seen, int32_t* __restrict__ n_scored, int Hkv, int budget, int rho) {
  const int b = blockIdx.x / Hkv, h = blockIdx.x - b * Hkv;
  const int64_t head = (int64_t)b * Hkv + h;
  const int N = P.n_old[b], wo = P.w_old[b], F = P.prefix[b];
  const int pad = F - old_count[head];
  const int cnt = ret_count[head];
  for (int i = threadIdx.x; i < cnt; i += 256) {
    const int e = ret_pos[head * budget + i];
    P.local_pos[head * budget + i] = e - F;
    ret_pos[head * budget + i] = e < F ? P.sorted_pos[head * budget + (e - pad)] : N - wo + (e - F);
  }
  if (h == 0 && threadIdx.x == 0) {
    const int total = N + (cu_new[b + 1] - cu_new[b]);
    n_seen[b] = total;
    n_scored[b] = total > rho ? total - rho : 0;
  }
}

size_t up256(size_t x) { return (x + 255) / 256 * 256; }

}  // namespace

// Upper bound of the extended tokens of all sequences (the true total depends on device-side state).
int64_t append_ext_tokens(const ltea_cfg& cfg, int n_seqs, int64_t total_new) {
  return (int64_t)n_seqs * ((int64_t)cfg.budget + 2 * (int64_t)cfg.window) + total_new;
}

size_t append_workspace(const ltea_cfg& cfg, int n_seqs, int64_t total_new, bool feature_keys) {
  const int64_t ext = append_ext_tokens(cfg, n_seqs, total_new);
  const size_t esz = cfg.dtype == LTEA_F32 ? 4 : 2;
  size_t b = 0;
  b += 7 * up256(sizeof(int32_t) * (size_t)(n_seqs + 1));                                 // per-sequence plan arrays
  b += 4 * up256(sizeof(int32_t) * (size_t)n_seqs * cfg.Hkv * (size_t)(cfg.budget > 0 ? cfg.budget : 1));  // sorted_pos, sorted_slot, local_pos, old counts
  b += (feature_keys ? 3 : 2) * up256((size_t)ext * cfg.Hkv * cfg.D * esz);                 // extended K, V (, scoring keys)
  b += up256((size_t)ext * cfg.Hkv * sizeof(float));                                        // extended logits / keys
  return b;
}

// Carves the workspace; returns the bytes used.  `ext_k`, `ext_v`, `ext_logits`, `old_count` receive the buffers.
static size_t carve(const ltea_cfg& cfg, int n_seqs, int64_t total_new, char* ws, AppendPlan& P, char*& ext_k,
                    char*& ext_v, float*& ext_logits, int32_t*& old_count) {
  const int64_t ext = append_ext_tokens(cfg, n_seqs, total_new);
  const size_t esz = cfg.dtype == LTEA_F32 ? 4 : 2;
  uintptr_t p = reinterpret_cast<uintptr_t>(ws);   // integer arithmetic: a size query carves from a null base
  auto take = [&](size_t bytes) { char* r = reinterpret_cast<char*>(p); p += up256(bytes); return r; };
  const size_t per_seq = sizeof(int32_t) * (size_t)(n_seqs + 1);
  P.n_old = reinterpret_cast<int32_t*>(take(per_seq));
  P.w_old = reinterpret_cast<int32_t*>(take(per_seq));
  P.prefix = reinterpret_cast<int32_t*>(take(per_seq));
  P.cu_ext = reinterpret_cast<int32_t*>(take(per_seq));
  P.cu_score = reinterpret_cast<int32_t*>(take(per_seq));
  P.kv_start = reinterpret_cast<int32_t*>(take(per_seq));
  P.kv_len = reinterpret_cast<int32_t*>(take(per_seq));
  const size_t per_entry = sizeof(int32_t) * (size_t)n_seqs * cfg.Hkv * (size_t)(cfg.budget > 0 ? cfg.budget : 1);
  P.sorted_pos = reinterpret_cast<int32_t*>(take(per_entry));
  P.sorted_slot = reinterpret_cast<int32_t*>(take(per_entry));
  P.local_pos = reinterpret_cast<int32_t*>(take(per_entry));
  old_count = reinterpret_cast<int32_t*>(take(per_entry));
  ext_k = take((size_t)ext * cfg.Hkv * cfg.D * esz);
  ext_v = take((size_t)ext * cfg.Hkv * cfg.D * esz);
  ext_logits = reinterpret_cast<float*>(take((size_t)ext * cfg.Hkv * sizeof(float)));
  // an optional third key buffer (scoring keys) follows; launch_append_build takes it from here
  return (size_t)(p - reinterpret_cast<uintptr_t>(ws));
}

// Stage 1 of the continuation: plan, ranks, extended K/V.  Returns the device arrays later stages need.
// With `rope` or `kf_new` given, out->ext_kf is a third buffer with the keys as the scoring CNN wants them.
hipError_t launch_append_build(const ltea_cfg& cfg, const void* k_new, const void* v_new, const void* kf_new,
                               int64_t stride_tok, int64_t stride_head, const int32_t* cu_new, int n_seqs,
                               int64_t total_new, int32_t max_new, const ltea_rope* rope, int32_t* status,
                               const ltea_cache& c, void* workspace, AppendBuffers* out, hipStream_t stream) {
  AppendPlan P;
  char *ext_k, *ext_v;
  float* ext_logits;
  int32_t* old_count;
  const size_t used = carve(cfg, n_seqs, total_new, static_cast<char*>(workspace), P, ext_k, ext_v, ext_logits, old_count);
  const bool feature_keys = rope != nullptr || kf_new != nullptr;
  char* ext_kf = feature_keys ? static_cast<char*>(workspace) + used : nullptr;
  const int64_t esz = cfg.dtype == LTEA_F32 ? 4 : 2;
  const unsigned heads = (unsigned)n_seqs * (unsigned)cfg.Hkv;
  hipLaunchKernelGGL(append_plan_rank_kernel, dim3(1u + heads), dim3(256), 0, stream, P, cu_new, c.n_seen, n_seqs, cfg.window,
                     cfg.budget, c.ret_pos, c.ret_count, old_count);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  BuildArgs a;
  a.k_new = static_cast<const char*>(k_new); a.v_new = static_cast<const char*>(v_new);
  a.kf_new = static_cast<const char*>(kf_new);
  a.tok_bytes = stride_tok * esz; a.head_bytes = stride_head * esz; a.cu_new = cu_new;
  a.k_win = static_cast<const char*>(c.k_win); a.v_win = static_cast<const char*>(c.v_win);
  a.k_ret = static_cast<const char*>(c.k_ret); a.v_ret = static_cast<const char*>(c.v_ret);
  a.ret_count = c.ret_count; a.k_ext = ext_k; a.v_ext = ext_v; a.kf_ext = ext_kf;
  a.rope = rope_dev(rope); a.status = status;
  a.Hkv = cfg.Hkv; a.window = cfg.window; a.budget = cfg.budget; a.row_bytes = (int)(cfg.D * esz);
  out->max_ext_len = cfg.budget + 2 * cfg.window + max_new;
  const unsigned chunks = (unsigned)((out->max_ext_len + 127) / 128);
  if (cfg.dtype == LTEA_F32) hipLaunchKernelGGL(append_build_kernel<float>, dim3(heads, chunks), dim3(256), 0, stream, P, a);
  else hipLaunchKernelGGL(append_build_kernel<bf16_t>, dim3(heads, chunks), dim3(256), 0, stream, P, a);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  out->ext_k = ext_k; out->ext_v = ext_v; out->ext_kf = ext_kf != nullptr ? ext_kf : ext_k;
  out->ext_logits = ext_logits; out->cu_ext = P.cu_ext; out->cu_score = P.cu_score;
  out->kv_start = P.kv_start; out->kv_len = P.kv_len; out->local_pos = P.local_pos;
  out->total_ext = append_ext_tokens(cfg, n_seqs, total_new);
  return hipSuccess;
}

hipError_t launch_append_keys(const ltea_cfg& cfg, int n_seqs, int64_t total_new, const ltea_cache& c, int rho,
                              void* workspace, const AppendBuffers& buf, hipStream_t stream) {
  AppendPlan P;
  char *ext_k, *ext_v;
  float* ext_logits;
  int32_t* old_count;
  carve(cfg, n_seqs, total_new, static_cast<char*>(workspace), P, ext_k, ext_v, ext_logits, old_count);
  const unsigned heads = (unsigned)n_seqs * (unsigned)cfg.Hkv;
  const unsigned chunks = (unsigned)((buf.max_ext_len + 1023) / 1024);
  hipLaunchKernelGGL(append_keys_kernel, dim3(heads, chunks), dim3(256), 0, stream, P, ext_logits, buf.total_ext,
                     c.win_score, c.ret_score, c.ret_count, cfg.Hkv, cfg.window, cfg.budget, cfg.sink, rho);
  return hipGetLastError();
}

hipError_t launch_append_fixup(const ltea_cfg& cfg, const int32_t* cu_new, int n_seqs, int64_t total_new,
                               const ltea_cache& c, int rho, void* workspace, hipStream_t stream) {
  AppendPlan P;
  char *ext_k, *ext_v;
  float* ext_logits;
  int32_t* old_count;
  carve(cfg, n_seqs, total_new, static_cast<char*>(workspace), P, ext_k, ext_v, ext_logits, old_count);
  const unsigned heads = (unsigned)n_seqs * (unsigned)cfg.Hkv;
  hipLaunchKernelGGL(append_fixup_kernel, dim3(heads), dim3(256), 0, stream, P, cu_new, c.ret_pos, c.ret_count, old_count,
                     c.n_seen, c.n_scored, cfg.Hkv, cfg.budget > 0 ? cfg.budget : 1, rho);
  return hipGetLastError();
}

}  // namespace ltea
