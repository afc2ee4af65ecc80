// Inverse rotary embedding of cached keys on the device (paper Section 3.1.3, lazy scoring paragraph: the cache holds
// the keys after the rotation, the scoring CNN wants them as they were before it, so they are rotated back with the
// model's cached sinusoids and negated sines).  Shared by the batched scoring of the decode ring and by the
// continuation of a prefill.
#pragma once
#include "ltea_common.h"

namespace ltea {

struct RopeDev {
  const float *cos, *sin;   // [n_pos][rot_dim / 2]
  int n_pos, rot_dim, interleaved;
};

inline RopeDev rope_dev(const ltea_rope* rope) {
  return RopeDev{rope ? rope->cos : nullptr, rope ? rope->sin : nullptr, rope ? rope->n_pos : 0,
                 rope ? rope->rot_dim : 0, rope ? rope->interleaved : 0};
}

template <typename T> struct Elems;   // 16 bytes <-> fp32 values
template <> struct Elems<float> {
  static constexpr int N = 4;
  static __device__ __forceinline__ void unpack(const u32x4& r, float (&x)[4]) {
#pragma unroll
    for (int i = 0; i < 4; ++i) x[i] = __uint_as_float(r[i]);
  }
  static __device__ __forceinline__ u32x4 pack(const float (&x)[4]) {
    return u32x4{__float_as_uint(x[0]), __float_as_uint(x[1]), __float_as_uint(x[2]), __float_as_uint(x[3])};
  }
};
template <> struct Elems<bf16_t> {
  static constexpr int N = 8;
  static __device__ __forceinline__ void unpack(const u32x4& r, float (&x)[8]) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      x[2 * i] = __uint_as_float(r[i] << 16);
      x[2 * i + 1] = __uint_as_float(r[i] & 0xFFFF0000u);
    }
  }
  static __device__ __forceinline__ u32x4 pack(const float (&x)[8]) {
    u32x4 r;
#pragma unroll
    for (int i = 0; i < 4; ++i)
      r[i] = (uint32_t)__builtin_bit_cast(uint16_t, from_f32<bf16_t>(x[2 * i])) |
             ((uint32_t)__builtin_bit_cast(uint16_t, from_f32<bf16_t>(x[2 * i + 1])) << 16);
    return r;
  }
};

// The 16-byte piece starting at element e0 of the key row `row` (the row as cached, i.e. rotated at position p),
// rotated back and rounded to the storage type.  `piece` is that piece as already loaded.  Elements at or beyond
// rot_dim pass through.  The caller has checked p < rope.n_pos.
// Inverse rotation of the pair (a, b): (a cos + b sin, -a sin + b cos).
template <typename T>
__device__ __forceinline__ u32x4 unrotate_piece(const RopeDev& rope, int p, int e0, const u32x4& piece, const T* row) {
  constexpr int EPP = Elems<T>::N;
  if (e0 >= rope.rot_dim) return piece;
  const int half = rope.rot_dim / 2;
  const float* ct = rope.cos + (int64_t)p * half;
  const float* st = rope.sin + (int64_t)p * half;
  float x[EPP], y[EPP];
  Elems<T>::unpack(piece, x);
  if (rope.interleaved) {
#pragma unroll
    for (int j = 0; j < EPP; j += 2) {
      const float c = ct[(e0 + j) / 2], s = st[(e0 + j) / 2];
      y[j] = fmaf(x[j + 1], s, x[j] * c);
      y[j + 1] = fmaf(x[j + 1], c, -(x[j] * s));
    }
  } else {
    const bool is_b = e0 >= half;                       // this piece holds the second members of its pairs
    const int partner = is_b ? e0 - half : e0 + half;
    float o[EPP];
    Elems<T>::unpack(*reinterpret_cast<const u32x4*>(row + partner), o);
    const int i0 = is_b ? e0 - half : e0;
#pragma unroll
    for (int j = 0; j < EPP; ++j) {
      const float c = ct[i0 + j], s = st[i0 + j];
      y[j] = is_b ? fmaf(x[j], c, -(o[j] * s)) : fmaf(o[j], s, x[j] * c);
    }
  }
  return Elems<T>::pack(y);
}

}  // namespace ltea
