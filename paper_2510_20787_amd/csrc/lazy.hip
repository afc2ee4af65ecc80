// Deferred, batched scoring of the decode cache (paper Section 3.1.3, lazy scoring paragraph).
//
// Between decode steps that do not score, the logits of all positions n_scored .. n_seen - rho - 1 of every sequence
// are produced at once: the ring rows those positions' receptive fields cover are packed in position order (the
// paper's "rotate the buffer"), the cached keys are optionally rotated back with the model's cached sinusoids and
// negated sines (the cache holds post-rotation keys, the scoring CNN wants them as they were before), the prefill
// scoring kernels run over the packed rows, and the new logits are scattered into win_score.
//
//   rescore_pack_kernel     grid (sequence, row chunk).  Sequence b owns rows b*window .. (b+1)*window - 1 of the
//                           packed buffers (fixed slots, so no prefix sum over the batch): row r holds position
//                           lo + r, lo = max(0, n_scored - rho); rows past the newest token are zero and are never
//                           inside the receptive field of a logit that is read back.  Also writes the per-sequence
//                           plan (lo, first new, end new) and the cu_seqlens of the fixed slots.
//   (scoring)               any of the prefill scoring launchers over B sequences of `window` rows.
//   rescore_scatter_kernel  one workgroup per sequence: logits of the newly final positions -> win_score,
//                           n_scored = n_seen - rho.
//
// A slot whose left edge is not the sequence start yields wrong logits for its first rho rows (the kernels pad
// there); those rows are the left context of the first unscored position and are not read back.
#include "ltea_common.h"
#include "ltea_kernels.h"
#include "rope_dev.h"

namespace ltea {
namespace {

struct PackArgs {
  const void *k_win, *v_win;
  const int32_t *n_seen, *n_scored;
  void *pk, *pv;
  int32_t *cu, *plan, *status;
  int B, Hkv, D, window, rho, rows_per_block;
  RopeDev rope;
};

template <typename T>
__global__ void __launch_bounds__(256)
rescore_pack_kernel(PackArgs A) {
  constexpr int EPP = Elems<T>::N;
  const int b = blockIdx.x;
  const int window = A.window, Hkv = A.Hkv, D = A.D, rho = A.rho;
  const int n = A.n_seen[b];
  const int first_new = A.n_scored[b];
  const int end_new = n - rho;
  const bool any = end_new > first_new;
  int lo = first_new - rho > 0 ? first_new - rho : 0;
  const int ring_lo = n - window > 0 ? n - window : 0;
  bool late = false;
  if (any && lo < ring_lo) { late = true; lo = ring_lo; }   // left context already overwritten: flagged below
  const int len = any ? n - lo : 0;
  if (blockIdx.y == 0 && threadIdx.x == 0) {
    A.plan[3 * b] = lo;
    // positions below lo (only when late) have no ring row any more: nothing is read back for them
    const int first_read = first_new > lo ? first_new : lo;
    A.plan[3 * b + 1] = first_read;
    A.plan[3 * b + 2] = any ? end_new : first_read;
    A.cu[b] = b * window;
    if (b == A.B - 1) A.cu[A.B] = A.B * window;
    if (late && A.status != nullptr) atomicOr(A.status, LTEA_LATE_SCORING);
  }
  const int pieces = D / EPP;
  const int r_begin = blockIdx.y * A.rows_per_block;
  const int r_end = r_begin + A.rows_per_block < window ? r_begin + A.rows_per_block : window;
  const int items = (r_end - r_begin) * Hkv * pieces;
  const T* kw = static_cast<const T*>(A.k_win);
  const T* vw = static_cast<const T*>(A.v_win);
  T* pk = static_cast<T*>(A.pk);
  T* pv = static_cast<T*>(A.pv);
  const int rot = A.rope.cos != nullptr ? A.rope.rot_dim : 0;
  bool out_of_tables = false;
  for (int i = threadIdx.x; i < items; i += 256) {
    const int pc = i % pieces, h = (i / pieces) % Hkv, r = r_begin + i / (pieces * Hkv);
    const int64_t dst = (((int64_t)b * window + r) * Hkv + h) * D + pc * EPP;
    u32x4 kraw = {0u, 0u, 0u, 0u}, vraw = {0u, 0u, 0u, 0u};
    if (r < len) {
      const int p = lo + r;
      const int64_t src = (((int64_t)b * Hkv + h) * window + p % window) * D;
      kraw = *reinterpret_cast<const u32x4*>(kw + src + pc * EPP);
      vraw = *reinterpret_cast<const u32x4*>(vw + src + pc * EPP);
      if (pc * EPP < rot) {
        if (p >= A.rope.n_pos) out_of_tables = true;
        else kraw = unrotate_piece<T>(A.rope, p, pc * EPP, kraw, kw + src);
      }
    }
    *reinterpret_cast<u32x4*>(pk + dst) = kraw;
    *reinterpret_cast<u32x4*>(pv + dst) = vraw;
  }
  if (out_of_tables && A.status != nullptr) atomicOr(A.status, LTEA_ROPE_RANGE);
}

__global__ void __launch_bounds__(256)
rescore_scatter_kernel(const float* __restrict__ logits, const int32_t* __restrict__ plan, float* __restrict__ win_score,
                       int32_t* __restrict__ n_scored, int B, int Hkv, int window) {
  const int b = blockIdx.x;
  const int lo = plan[3 * b], first_new = plan[3 * b + 1], end_new = plan[3 * b + 2];
  const int count = end_new - first_new;
  const int64_t total = (int64_t)B * window;
  for (int i = threadIdx.x; i < count * Hkv; i += 256) {
    const int h = i / count, j = first_new + (i - h * count);
    win_score[((int64_t)b * Hkv + h) * window + j % window] = logits[(int64_t)h * total + (int64_t)b * window + (j - lo)];
  }
  if (threadIdx.x == 0 && count > 0) n_scored[b] = end_new;
}

size_t up256(size_t x) { return (x + 255) / 256 * 256; }

}  // namespace

size_t rescore_workspace(const ltea_cfg& cfg, int n_seqs, RescoreBuffers* out, void* base) {
  const size_t esz = cfg.dtype == LTEA_F32 ? 4 : 2;
  const size_t rows = (size_t)n_seqs * cfg.window;
  uintptr_t p = reinterpret_cast<uintptr_t>(base);   // integer arithmetic: a size query carves from a null base
  auto take = [&](size_t bytes) { char* r = reinterpret_cast<char*>(p); p += up256(bytes); return r; };
  void* pk = take(rows * cfg.Hkv * cfg.D * esz);
  void* pv = take(rows * cfg.Hkv * cfg.D * esz);
  float* lg = reinterpret_cast<float*>(take(rows * cfg.Hkv * sizeof(float)));
  int32_t* cu = reinterpret_cast<int32_t*>(take(((size_t)n_seqs + 1) * sizeof(int32_t)));
  int32_t* plan = reinterpret_cast<int32_t*>(take((size_t)n_seqs * 3 * sizeof(int32_t)));
  if (out) { out->pk = pk; out->pv = pv; out->logits = lg; out->cu = cu; out->plan = plan; out->total = (int64_t)rows; }
  return (size_t)(p - reinterpret_cast<uintptr_t>(base));
}

hipError_t launch_rescore_pack(const ltea_cfg& cfg, const ltea_rope* rope, const ltea_cache& c, int n_seqs, int rho,
                               int32_t* status, const RescoreBuffers& buf, hipStream_t stream) {
  PackArgs A;
  A.k_win = c.k_win; A.v_win = c.v_win; A.n_seen = c.n_seen; A.n_scored = c.n_scored;
  A.pk = buf.pk; A.pv = buf.pv; A.cu = buf.cu; A.plan = buf.plan; A.status = status;
  A.B = n_seqs; A.Hkv = cfg.Hkv; A.D = cfg.D; A.window = cfg.window; A.rho = rho;
  A.rows_per_block = 32;
  A.rope = rope_dev(rope);
  const dim3 grid((unsigned)n_seqs, (unsigned)((cfg.window + A.rows_per_block - 1) / A.rows_per_block));
  if (cfg.dtype == LTEA_F32) hipLaunchKernelGGL(rescore_pack_kernel<float>, grid, dim3(256), 0, stream, A);
  else hipLaunchKernelGGL(rescore_pack_kernel<bf16_t>, grid, dim3(256), 0, stream, A);
  return hipGetLastError();
}

hipError_t launch_rescore_scatter(const ltea_cfg& cfg, const ltea_cache& c, int n_seqs, const RescoreBuffers& buf,
                                  hipStream_t stream) {
  hipLaunchKernelGGL(rescore_scatter_kernel, dim3((unsigned)n_seqs), dim3(256), 0, stream, buf.logits, buf.plan,
                     c.win_score, c.n_scored, n_seqs, cfg.Hkv, cfg.window);
  return hipGetLastError();
}

}  // namespace ltea
