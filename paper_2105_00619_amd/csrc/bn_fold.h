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
#pragma unroll
  for (int k = 0; k < EV; ++k) {
    const float y = bn_affine(to_f32(t.v[k]), sc[k], sh[k]);
    t.v[k] = from_f32<T>(relu ? fmaxf(y, 0.f) : y);
  }
  return __builtin_bit_cast(Chunk, t);
}

}  // namespace oseq
