// Pieces shared by the scoring kernels that keep their conv weights in registers and load token tiles from global
// memory straight into LDS (paper Section 3.1.1; Appendix A).
#pragma once
#include "ltea_common.h"
#include "ltea_kernels.h"

namespace ltea {

// 16 bytes per lane from a buffer straight into LDS: lane l's piece lands at lds_addr + 16 * l.
__device__ __forceinline__ void dma16(u32x4 rsrc, uint32_t lds_addr, uint32_t voff) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
               :: "s"(lds_addr), "v"(voff), "s"(rsrc) : "memory");
}
// s_waitcnt vmcnt(0) through the builtin, so that the compiler's own wait-count bookkeeping sees it (it cannot see
// into the asm statement above).
__device__ __forceinline__ void wait_loads() {
  __builtin_amdgcn_s_waitcnt(0x0F70);
  asm volatile("" ::: "memory");
}
// s_waitcnt vmcnt(N) for the depths a pipeline needs besides 0 (the immediate has to be a constant; the other
// counters stay at their maxima = not waited for; vmcnt's upper two bits sit in bits 15:14)
template <int N> __device__ __forceinline__ void wait_loads_but() {
  static_assert(N > 0 && N < 64, "vmcnt is a 6-bit counter");
  __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
  asm volatile("" ::: "memory");
}

// Buffer descriptor (raw, 32-bit offsets, out-of-range reads give zeros) over `bytes` bytes at `p`, in scalar registers.
__device__ __forceinline__ u32x4 make_raw_rsrc(const void* p, uint32_t bytes) {
  const uint64_t a = reinterpret_cast<uint64_t>(p);
  u32x4 r;
  r[0] = __builtin_amdgcn_readfirstlane((uint32_t)a);
  r[1] = __builtin_amdgcn_readfirstlane((uint32_t)(a >> 32) & 0xFFFFu);
  r[2] = __builtin_amdgcn_readfirstlane(bytes);
  r[3] = 0x00020000u;
  return r;
}

// y * sigmoid(y) with the hardware's exp2 and reciprocal (1 ulp each)
__device__ __forceinline__ float silu_fast(float y) {
  return y * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.44269504f * y));
}

// Consecutive tiles per workgroup for a kernel that runs one workgroup per CU (256 of them): the number that makes the
// launch shortest when a workgroup costs its tiles plus about three tiles' worth of start-up and the grid runs in
// rounds of 256 workgroups.  The count of groups is exact for a batch of equal lengths, an upper bound otherwise.
inline int pick_group_tiles(const SeqView& sv, int Hkv, int tile_tokens, int max_tiles) {
  int best = 1;
  int64_t best_cost = -1;
  for (int g = 1; g <= max_tiles; ++g) {
    const int64_t span = (int64_t)g * tile_tokens;
    const int64_t groups = (int64_t)sv.n_seqs * sv.max_seqlen == sv.total_tokens
                               ? (int64_t)sv.n_seqs * ((sv.max_seqlen + span - 1) / span)
                               : sv.total_tokens / span + sv.n_seqs;
    const int64_t rounds = (groups * Hkv + 255) / 256;
    const int64_t cost = rounds * (g + 3);
    if (best_cost < 0 || cost < best_cost) { best_cost = cost; best = g; }
  }
  return best;
}

}  // namespace ltea
