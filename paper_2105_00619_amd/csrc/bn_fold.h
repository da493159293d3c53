// Operand-side BatchNorm for the convolution kernels that read z in place of the activation.
#pragma once
#include "dev_common.h"

namespace oseq {

// BatchNorm apply (+ReLU) on 16 bytes of z held in registers: the values the stand-alone apply kernel stores (the same
// arithmetic, one rounding), for kernels that read z in place of the activation.  sc / sh: scale and shift of the piece's
// 16 / sizeof(T) channels.
template <class T>
__device__ __forceinline__ Chunk bn_fold_chunk(const Chunk& c, const float (&sc)[16 / sizeof(T)],
                                               const float (&sh)[16 / sizeof(T)], int relu) {
  constexpr int EV = 16 / (int)sizeof(T);
  Vec<T, EV> t = __builtin_bit_cast(Vec<T, EV>, c);
  float y[EV];
#pragma unroll
  for (int k = 0; k < EV; ++k) {
    const float v = bn_affine(to_f32(t.v[k]), sc[k], sh[k]);
    y[k] = relu ? fmaxf(v, 0.f) : v;
  }
  if constexpr (sizeof(T) == 2) {
#pragma unroll
    for (int k = 0; k < EV; k += 2) {
      const typename Pair16<T>::V q = from_f32x2<T>(y[k], y[k + 1]);
      t.v[k] = q[0]; t.v[k + 1] = q[1];
    }
  } else {
#pragma unroll
    for (int k = 0; k < EV; ++k) t.v[k] = from_f32<T>(y[k]);
  }
  return __builtin_bit_cast(Chunk, t);
}

// The same with the ReLU flag known at compile time, for callers that branch on it once per tile.
template <class T, bool RELU>
__device__ __forceinline__ Chunk bn_fold_chunk_t(const Chunk& c, const float (&sc)[16 / sizeof(T)],
                                                 const float (&sh)[16 / sizeof(T)]) {
  constexpr int EV = 16 / (int)sizeof(T);
  Vec<T, EV> t = __builtin_bit_cast(Vec<T, EV>, c);
  float y[EV];
#pragma unroll
  for (int k = 0; k < EV; ++k) {
    const float v = bn_affine(to_f32(t.v[k]), sc[k], sh[k]);
    y[k] = RELU ? fmaxf(v, 0.f) : v;
  }
  if constexpr (sizeof(T) == 2) {
#pragma unroll
    for (int k = 0; k < EV; k += 2) {
      const typename Pair16<T>::V q = from_f32x2<T>(y[k], y[k + 1]);
      t.v[k] = q[0]; t.v[k + 1] = q[1];
    }
  } else {
#pragma unroll
    for (int k = 0; k < EV; ++k) t.v[k] = from_f32<T>(y[k]);
  }
  return __builtin_bit_cast(Chunk, t);
}

}  // namespace oseq
