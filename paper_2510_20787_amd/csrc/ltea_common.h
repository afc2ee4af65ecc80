// Device-side helpers shared by the gfx950 kernels of libltea (wave64 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ltea {

constexpr int kWave = 64;

typedef __bf16 bf16_t;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

__device__ __forceinline__ float to_f32(float x) { return x; }
__device__ __forceinline__ float to_f32(bf16_t x) { return static_cast<float>(x); }
__device__ __forceinline__ float bf16_bits_to_f32(uint32_t bits16) { return __uint_as_float(bits16 << 16); }

template <typename T> __device__ __forceinline__ T from_f32(float x);
template <> __device__ __forceinline__ float from_f32<float>(float x) { return x; }
template <> __device__ __forceinline__ bf16_t from_f32<bf16_t>(float x) { return static_cast<bf16_t>(x); }  // RNE

// Swish with beta = 1 in fp32.
__device__ __forceinline__ float silu_f32(float x) { return x / (1.0f + expf(-x)); }

// Monotone map float -> uint32: a < b (as floats, -0 < +0) <=> key(a) < key(b). NaNs are never passed in.
__device__ __forceinline__ uint32_t order_key(float x) {
  uint32_t u = __float_as_uint(x);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// Canonical selection key of a token: +inf for sinks, else the logit with -0 folded to +0 so that
// equal floats have equal integer keys.
__device__ __forceinline__ float select_key(float z, int pos, int sink) {
  if (pos < sink) return __uint_as_float(0x7F800000u);
  return z + 0.0f;
}

__device__ __forceinline__ float wave_max(float x) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) x = fmaxf(x, __shfl_xor(x, off, kWave));
  return x;
}
__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) x += __shfl_xor(x, off, kWave);
  return x;
}
__device__ __forceinline__ int wave_sum_i(int x) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) x += __shfl_xor(x, off, kWave);
  return x;
}

// Index s of the sequence holding packed token t: cu[s] <= t < cu[s+1]. Empty sequences are skipped.
__device__ __forceinline__ int find_sequence(const int32_t* __restrict__ cu, int n_seqs, int64_t t) {
  int lo = 0, hi = n_seqs;  // invariant: cu[lo] <= t < cu[hi]
  while (hi - lo > 1) {
    int mid = (lo + hi) >> 1;
    if (cu[mid] <= t) lo = mid; else hi = mid;
  }
  return lo;
}

// Which sequence owns flat tile `flat`, when sequence i owns ceil(len_i / tile_len) consecutive tiles?  Called by
// every lane of a wave with the same arguments (full exec).  The lengths are read 64 sequences at a time with one
// vector load each for cu[i] and cu[i+1] and resolved with a wave prefix sum, so the search costs one trip to
// memory per 64 sequences instead of one per sequence.  Returns false if `flat` is past the last tile.
__device__ __forceinline__ bool locate_tile(const int32_t* __restrict__ cu, int n_seqs, int tile_len, int flat,
                                            int& seq, int& tile, int& lo, int& len) {
  const int lane = threadIdx.x & (kWave - 1);
  int before = 0;   // tiles owned by the sequences of earlier rounds
  for (int s0 = 0; s0 < n_seqs; s0 += kWave) {
    const int i = s0 + lane;
    const int ic = i < n_seqs ? i : n_seqs - 1;      // unconditional loads, inactive lanes count zero tiles
    const int a = cu[ic], b = cu[ic + 1];
    const int nt = i < n_seqs ? (b - a + tile_len - 1) / tile_len : 0;
    int inc = nt;
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
      const int t = __shfl_up(inc, off, kWave);
      if (lane >= off) inc += t;
    }
    const int total = __builtin_amdgcn_readfirstlane(__shfl(inc, kWave - 1, kWave));
    if (flat < before + total) {
      const unsigned long long m = __builtin_amdgcn_ballot_w64(inc > flat - before);
      const int l = __builtin_ctzll(m);
      // the results are wave-uniform: hand them back in scalar registers so that everything derived from them
      // (loop bounds, buffer descriptors) stays scalar
      seq = s0 + l;
      lo = __builtin_amdgcn_readfirstlane(__shfl(a, l, kWave));
      len = __builtin_amdgcn_readfirstlane(__shfl(b, l, kWave)) - lo;
      tile = flat - before -
             __builtin_amdgcn_readfirstlane(__shfl(inc, l, kWave) - __shfl(nt, l, kWave));
      return true;
    }
    before += total;
  }
  return false;
}

// The same enumeration in two parts: first every sequence's tiles from index `first_late` on, then the tiles before it
// (the first tiles of a sequence see a window that is still filling: a kernel whose work per tile grows with the number
// of keys in reach puts them last, where they fill the gaps that the long tiles leave when the grid drains).  The
// counts of flat indices are the same as locate_tile's: ceil(len / tile_len) per sequence.
__device__ __forceinline__ bool locate_tile_late_first(const int32_t* __restrict__ cu, int n_seqs, int tile_len,
                                                       int first_late, int flat, int& seq, int& tile, int& lo, int& len) {
  const int lane = threadIdx.x & (kWave - 1);
#pragma unroll 1
  for (int part = 0; part < 2; ++part) {
    for (int s0 = 0; s0 < n_seqs; s0 += kWave) {
      const int i = s0 + lane;
      const int ic = i < n_seqs ? i : n_seqs - 1;
      const int a = cu[ic], b = cu[ic + 1];
      const int all = i < n_seqs ? (b - a + tile_len - 1) / tile_len : 0;
      const int early = all < first_late ? all : first_late;
      const int nt = part == 0 ? all - early : early;
      int inc = nt;
#pragma unroll
      for (int off = 1; off < kWave; off <<= 1) {
        const int t = __shfl_up(inc, off, kWave);
        if (lane >= off) inc += t;
      }
      const int total = __builtin_amdgcn_readfirstlane(__shfl(inc, kWave - 1, kWave));
      if (flat < total) {
        const unsigned long long m = __builtin_amdgcn_ballot_w64(inc > flat);
        const int l = __builtin_ctzll(m);
        seq = s0 + l;
        lo = __builtin_amdgcn_readfirstlane(__shfl(a, l, kWave));
        len = __builtin_amdgcn_readfirstlane(__shfl(b, l, kWave)) - lo;
        const int within = flat - __builtin_amdgcn_readfirstlane(__shfl(inc, l, kWave) - __shfl(nt, l, kWave));
        const int early_l = __builtin_amdgcn_readfirstlane(__shfl(early, l, kWave));
        tile = part == 0 ? early_l + within : within;
        return true;
      }
      flat -= total;
    }
  }
  return false;
}

}  // namespace ltea
