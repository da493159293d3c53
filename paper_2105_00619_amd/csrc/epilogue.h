// Store half of the convolution kernels' epilogue, shared by the GEMM-shaped kernels.
//
// The accumulators of HR block rows lie in LDS as fp32 [HR][BN + 4].  Every one of the block's NT threads (256 unless
// the _nt form is used) handles, for HR * (BN / 8) / NT rows, 8 consecutive channels: bias / residual addend / ReLU in fp32, one rounding, one 16-byte (fp32: two) store,
// and optionally adds what it stored to its per-channel sum and sum of squares (the BatchNorm statistics).
//
// Loads and stores share one in-order counter on this hardware, so a load issued after a store cannot be waited for
// without waiting for the store.  Hence: all loads of a pass (bias, addends) are issued before its first store, and
// the (bias, addend) combinations are separate straight-line code paths chosen by a uniform branch, so that the
// common path without either contains no load at all and its stores are never waited for.
#pragma once
#include "dev_common.h"

namespace oseq {

typedef __attribute__((ext_vector_type(4))) float epi_v4f;

// rowoff(row): element offset of block row `row`'s first channel in the output tensor, or -1 if the row is not stored
// amask (with an addend; may be null): ReLU decisions as bits, byte e / V for the V = 16 / sizeof(T) elements from
// element offset e of the addend; an addend element whose bit is clear counts as zero.
template <int NT, class T, int BN, int HR, bool HB, bool HA, bool STAT, class RowOff>
__device__ __forceinline__ void epi_store_rows_nt(const float* ep, int tid, int n0, const float* __restrict__ bias,
                                               const T* __restrict__ addend, const uint8_t* __restrict__ amask,
                                               T* __restrict__ out, int relu, RowOff rowoff,
                                               float (&ss)[8], float (&qq)[8]) {
  constexpr int EP_PITCH = BN + 4;
  constexpr int GROUPS = BN / 8;                // 8-channel groups per row
  constexpr int PER_THREAD = HR * GROUPS / NT;  // rows per thread
  constexpr int RG = NT / GROUPS;               // rows between a thread's rows
  static_assert(PER_THREAD >= 1, "fewer rows than the block covers");
  const int c8 = (tid % GROUPS) * 8, erow = tid / GROUPS;
  const int col = n0 + c8;
  int64_t ro[PER_THREAD];
#pragma unroll
  for (int it = 0; it < PER_THREAD; ++it) ro[it] = rowoff(erow + it * RG);
  float bv[8];
  if (HB) {
#pragma unroll
    for (int k = 0; k < 8; ++k) bv[k] = bias[col + k];
  }
  Vec<T, 8> ad[PER_THREAD];
  unsigned mb[PER_THREAD];
  if (HA) {  // rows that are not stored read the tensor's first row
#pragma unroll
    for (int it = 0; it < PER_THREAD; ++it)
      ad[it] = *reinterpret_cast<const Vec<T, 8>*>(addend + (ro[it] >= 0 ? ro[it] : 0) + col);
#pragma unroll
    for (int it = 0; it < PER_THREAD; ++it) {
      mb[it] = 0xffu;
      if (amask) {
        const int64_t e = (ro[it] >= 0 ? ro[it] : 0) + col;
        if (sizeof(T) == 2) mb[it] = amask[e >> 3];
        else mb[it] = (amask[e >> 2] & 15u) | ((unsigned)(amask[(e >> 2) + 1] & 15u) << 4);
      }
    }
  }
  constexpr bool PAIRS = sizeof(T) == 2 && PER_THREAD % 2 == 0;
  Vec<T, 8> tv[STAT && PAIRS ? PER_THREAD : 1];
  // straight-line code for all rows (only the store is predicated), so that the LDS reads of the later rows are issued
  // while the earlier ones are converted
#pragma unroll
  for (int it = 0; it < PER_THREAD; ++it) {
    const int row = erow + it * RG;
    const epi_v4f x0 = *reinterpret_cast<const epi_v4f*>(&ep[row * EP_PITCH + c8]);
    const epi_v4f x1 = *reinterpret_cast<const epi_v4f*>(&ep[row * EP_PITCH + c8 + 4]);
    float v[8] = {x0[0], x0[1], x0[2], x0[3], x1[0], x1[1], x1[2], x1[3]};
    if (HB) {
#pragma unroll
      for (int k = 0; k < 8; ++k) v[k] += bv[k];
    }
    if (HA) {
#pragma unroll
      for (int k = 0; k < 8; ++k) v[k] += ((mb[it] >> k) & 1u) ? to_f32(ad[it].v[k]) : 0.f;
    }
    if (relu) {
#pragma unroll
      for (int k = 0; k < 8; ++k) v[k] = fmaxf(v[k], 0.f);
    }
    const Vec<T, 8> t = round_vec<T, 8>(v);
    if (ro[it] >= 0) *reinterpret_cast<Vec<T, 8>*>(out + ro[it] + col) = t;
    if constexpr (STAT && PAIRS) {
      tv[it] = t;
      if (ro[it] < 0) tv[it] = Vec<T, 8>{};  // a row that is not stored counts as zero
    } else if (STAT) {
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        const float r = ro[it] >= 0 ? to_f32(t.v[k]) : 0.f;
        ss[k] += r; qq[k] = __fmaf_rn(r, r, qq[k]);
      }
    }
  }
  // 16-bit types: two rows of a channel as one pair, its sum and its sum of squares one dot-product instruction each
  // (exact products, fp32 sum) instead of four operations per element
  if constexpr (STAT && PAIRS) {
    typedef typename Dot2<T>::V T2;
    T2 one2;
    one2[0] = from_f32<T>(1.f); one2[1] = from_f32<T>(1.f);
#pragma unroll
    for (int it = 0; it < PER_THREAD; it += 2)
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        T2 p2;
        p2[0] = tv[it].v[k]; p2[1] = tv[it + 1].v[k];
        ss[k] = Dot2<T>::run(p2, one2, ss[k]);
        qq[k] = Dot2<T>::run(p2, p2, qq[k]);
      }
  }
}

// The residual-adding pass in two halves, for a kernel whose block owns its CU alone and therefore has nobody to cover
// the latency of the addend loads: the addend pieces (and mask bytes) of a pass are requested one pass ahead
// (epi_load_addend_nt), before the stores of the pass in between, and added later (epi_store_rows_pre_nt).  Loads
// issued before stores can be waited for without waiting for those stores.
template <int NT, class T, int BN, int HR, class RowOff>
__device__ __forceinline__ void epi_load_addend_nt(int tid, int n0, const T* __restrict__ addend,
                                                   const uint8_t* __restrict__ amask, RowOff rowoff,
                                                   Vec<T, 8> (&ad)[HR * (BN / 8) / NT], unsigned (&mb)[HR * (BN / 8) / NT]) {
  constexpr int GROUPS = BN / 8, PER_THREAD = HR * GROUPS / NT, RG = NT / GROUPS;
  const int col = n0 + (tid % GROUPS) * 8, erow = tid / GROUPS;
#pragma unroll
  for (int it = 0; it < PER_THREAD; ++it) {
    const int64_t ro = rowoff(erow + it * RG);
    const int64_t e = (ro >= 0 ? ro : 0) + col;  // rows that are not stored read the tensor's first row
    if constexpr (sizeof(T) == 2) {  // read once, by this block only
      typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
      ad[it] = __builtin_bit_cast(Vec<T, 8>, __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(addend + e)));
    } else {
      ad[it] = *reinterpret_cast<const Vec<T, 8>*>(addend + e);
    }
    mb[it] = 0xffu;
    if (amask) {
      if (sizeof(T) == 2) mb[it] = amask[e >> 3];
      else mb[it] = (amask[e >> 2] & 15u) | ((unsigned)(amask[(e >> 2) + 1] & 15u) << 4);
    }
  }
}
template <int NT, class T, int BN, int HR, class RowOff>
__device__ __forceinline__ void epi_store_rows_pre_nt(const float* ep, int tid, int n0,
                                                      const Vec<T, 8> (&ad)[HR * (BN / 8) / NT],
                                                      const unsigned (&mb)[HR * (BN / 8) / NT], T* __restrict__ out,
                                                      RowOff rowoff) {
  constexpr int EP_PITCH = BN + 4;
  constexpr int GROUPS = BN / 8, PER_THREAD = HR * GROUPS / NT, RG = NT / GROUPS;
  const int c8 = (tid % GROUPS) * 8, erow = tid / GROUPS;
  const int col = n0 + c8;
#pragma unroll
  for (int it = 0; it < PER_THREAD; ++it) {
    const int row = erow + it * RG;
    const int64_t ro = rowoff(row);
    const epi_v4f x0 = *reinterpret_cast<const epi_v4f*>(&ep[row * EP_PITCH + c8]);
    const epi_v4f x1 = *reinterpret_cast<const epi_v4f*>(&ep[row * EP_PITCH + c8 + 4]);
    float v[8] = {x0[0], x0[1], x0[2], x0[3], x1[0], x1[1], x1[2], x1[3]};
#pragma unroll
    for (int k = 0; k < 8; ++k) v[k] += ((mb[it] >> k) & 1u) ? to_f32(ad[it].v[k]) : 0.f;
    const Vec<T, 8> t = round_vec<T, 8>(v);
    if (ro >= 0) *reinterpret_cast<Vec<T, 8>*>(out + ro + col) = t;
  }
}

// The uniform choice of the code path.  CAN_BIAS / CAN_ADD: whether the calling kernel is ever given a bias / an
// addend (forward kernels have no addend, data-gradient kernels no bias); the combinations that cannot occur are not
// compiled, which keeps their registers out of the kernel.
template <int NT, class T, int BN, int HR, bool CAN_BIAS, bool CAN_ADD, bool STAT, class RowOff>
__device__ __forceinline__ void epi_store_pass_nt(const float* ep, int tid, int n0, const float* __restrict__ bias,
                                                  const T* __restrict__ addend, const uint8_t* __restrict__ amask,
                                                  T* __restrict__ out, int relu, RowOff rowoff,
                                                  float (&ss)[8], float (&qq)[8]) {
  if (CAN_BIAS && bias) {
    if (CAN_ADD && addend) epi_store_rows_nt<NT, T, BN, HR, true, CAN_ADD, STAT>(ep, tid, n0, bias, addend, amask, out, relu, rowoff, ss, qq);
    else epi_store_rows_nt<NT, T, BN, HR, true, false, STAT>(ep, tid, n0, bias, addend, amask, out, relu, rowoff, ss, qq);
  } else {
    if (CAN_ADD && addend) epi_store_rows_nt<NT, T, BN, HR, false, true, STAT>(ep, tid, n0, bias, addend, amask, out, relu, rowoff, ss, qq);
    else epi_store_rows_nt<NT, T, BN, HR, false, false, STAT>(ep, tid, n0, bias, addend, amask, out, relu, rowoff, ss, qq);
  }
}
template <class T, int BN, int HR, bool CAN_BIAS, bool CAN_ADD, bool STAT, class RowOff>
__device__ __forceinline__ void epi_store_pass(const float* ep, int tid, int n0, const float* __restrict__ bias,
                                               const T* __restrict__ addend, const uint8_t* __restrict__ amask,
                                               T* __restrict__ out, int relu, RowOff rowoff,
                                               float (&ss)[8], float (&qq)[8]) {
  epi_store_pass_nt<256, T, BN, HR, CAN_BIAS, CAN_ADD, STAT>(ep, tid, n0, bias, addend, amask, out, relu, rowoff, ss, qq);
}

// raw fp32 sums of a depth range (no epilogue arithmetic): dst + rowoff(row) + channel
template <int BN, int HR, class RowOff>
__device__ __forceinline__ void epi_store_partial(const float* ep, int tid, int n0, float* __restrict__ dst, RowOff rowoff) {
  constexpr int EP_PITCH = BN + 4;
  constexpr int GROUPS = BN / 8;
  constexpr int PER_THREAD = HR * GROUPS / 256;
  constexpr int RG = 256 / GROUPS;
  const int c8 = (tid % GROUPS) * 8, erow = tid / GROUPS;
#pragma unroll
  for (int it = 0; it < PER_THREAD; ++it) {
    const int row = erow + it * RG;
    const int64_t ro = rowoff(row);
    if (ro < 0) continue;
    const epi_v4f x0 = *reinterpret_cast<const epi_v4f*>(&ep[row * EP_PITCH + c8]);
    const epi_v4f x1 = *reinterpret_cast<const epi_v4f*>(&ep[row * EP_PITCH + c8 + 4]);
    *reinterpret_cast<epi_v4f*>(dst + ro + n0 + c8) = x0;
    *reinterpret_cast<epi_v4f*>(dst + ro + n0 + c8 + 4) = x1;
  }
}

// Per-block channel sums from the threads' sums: the NT / (BN / 8) row groups of a channel are added in a fixed order
// through LDS (red: 2 * (NT / (BN / 8)) * BN floats, free to overwrite; called by all NT threads).
// dst_sum / dst_sq: this block's rows of the [blocks][2][channels] array, at the block's first channel.
template <int NT, int BN>
__device__ __forceinline__ void epi_stat_combine_nt(float* red, int tid, const float (&ss)[8], const float (&qq)[8],
                                                    float* __restrict__ dst_sum, float* __restrict__ dst_sq) {
  constexpr int GROUPS = BN / 8;
  constexpr int RG = NT / GROUPS;
  const int c8 = (tid % GROUPS) * 8, erow = tid / GROUPS;
  __syncthreads();
#pragma unroll
  for (int k = 0; k < 8; ++k) { red[erow * BN + c8 + k] = ss[k]; red[(RG + erow) * BN + c8 + k] = qq[k]; }
  __syncthreads();
  if (tid < BN) {
    float s0 = red[tid], q0 = red[RG * BN + tid];
#pragma unroll 8
    for (int r = 1; r < RG; ++r) { s0 += red[r * BN + tid]; q0 += red[(RG + r) * BN + tid]; }
    dst_sum[tid] = s0;
    dst_sq[tid] = q0;
  }
}
template <int BN>
__device__ __forceinline__ void epi_stat_combine(float* red, int tid, const float (&ss)[8], const float (&qq)[8],
                                                 float* __restrict__ dst_sum, float* __restrict__ dst_sq) {
  epi_stat_combine_nt<256, BN>(red, tid, ss, qq, dst_sum, dst_sq);
}

}  // namespace oseq
