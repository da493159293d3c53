// Operand-side BatchNorm for the convolution kernels that read z in place of the activation.
#pragma once
#include "dev_common.h"

namespace oseq {

// BatchNorm apply + ReLU on 16 bytes of z held in registers: the values the stand-alone apply kernel stores (the same
// arithmetic, one rounding), for kernels that read z in place of the activation.  sc / sh: scale and shift of the piece's
// 16 / sizeof(T) channels.  Only a BatchNorm that is followed by a ReLU is ever folded into its reader (the choice is
// made where the schedule is built), so the ReLU is not a flag here: in the inner loops of the matrix-core kernels a
// select per element costs as much as the ReLU itself.
template <class T>
__device__ __forceinline__ Chunk bn_fold_chunk(const Chunk& c, const float (&sc)[16 / sizeof(T)],
                                               const float (&sh)[16 / sizeof(T)]) {
  constexpr int EV = 16 / (int)sizeof(T);
  const Vec<T, EV> t = __builtin_bit_cast(Vec<T, EV>, c);
  float y[EV];
#pragma unroll
  for (int k = 0; k < EV; ++k) y[k] = fmaxf(bn_affine(to_f32(t.v[k]), sc[k], sh[k]), 0.f);
  return __builtin_bit_cast(Chunk, round_vec<T, EV>(y));
}

}  // namespace oseq
