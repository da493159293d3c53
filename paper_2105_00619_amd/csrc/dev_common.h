// Device-side helpers shared by the HIP kernels: storage types, conversions, vector loads.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kernels.h"
#include "launch.h"

namespace oseq {

typedef _Float16 f16_t;
typedef __bf16 bf16_t;

__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ float to_f32(f16_t v) { return (float)v; }
__device__ __forceinline__ float to_f32(bf16_t v) { return (float)v; }

template <class T> __device__ __forceinline__ T from_f32(float v);
template <> __device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ f16_t from_f32<f16_t>(float v) { return (f16_t)v; }    // round to nearest even
template <> __device__ __forceinline__ bf16_t from_f32<bf16_t>(float v) { return (bf16_t)v; }  // round to nearest even

// Two floats rounded (to nearest even) into a pair of 16-bit values in one register: one packed conversion instead of
// two conversions and a merge.
typedef __attribute__((ext_vector_type(2))) float f32x2_t;
template <class T> struct Pair16;
template <> struct Pair16<f16_t> { typedef __attribute__((ext_vector_type(2))) _Float16 V; };
template <> struct Pair16<bf16_t> { typedef __attribute__((ext_vector_type(2))) __bf16 V; };
template <class T> __device__ __forceinline__ typename Pair16<T>::V from_f32x2(float a, float b) {
  const f32x2_t v = {a, b};
  return __builtin_convertvector(v, typename Pair16<T>::V);
}

// sum of the two products of a pair of 16-bit values, added to c in fp32 (one instruction)
template <class T> struct Dot2;
template <> struct Dot2<bf16_t> {
  typedef __attribute__((ext_vector_type(2))) __bf16 V;
  __device__ static __forceinline__ float run(V a, V b, float c) { return __builtin_amdgcn_fdot2_f32_bf16(a, b, c, false); }
};
template <> struct Dot2<f16_t> {
  typedef __attribute__((ext_vector_type(2))) _Float16 V;
  __device__ static __forceinline__ float run(V a, V b, float c) { return __builtin_amdgcn_fdot2(a, b, c, false); }
};

// V consecutive elements of T, loaded and stored as one access.
template <class T, int V>
struct alignas(sizeof(T) * V) Vec {
  T v[V];
};

// the same as a streaming (non-temporal) load where the V elements are 16 bytes
template <class T, int V>
__device__ __forceinline__ void load_f32_nt(const T* p, float (&out)[V]) {
  if constexpr (sizeof(T) * V == 16) {
    typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
    const u32x4 c = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
    const Vec<T, V> t = __builtin_bit_cast(Vec<T, V>, c);
#pragma unroll
    for (int i = 0; i < V; ++i) out[i] = to_f32(t.v[i]);
  } else {
    Vec<T, V> t = *reinterpret_cast<const Vec<T, V>*>(p);
#pragma unroll
    for (int i = 0; i < V; ++i) out[i] = to_f32(t.v[i]);
  }
}
template <class T, int V>
__device__ __forceinline__ void load_f32(const T* p, float (&out)[V]) {
  Vec<T, V> t = *reinterpret_cast<const Vec<T, V>*>(p);
#pragma unroll
  for (int i = 0; i < V; ++i) out[i] = to_f32(t.v[i]);
}
// V floats rounded to T (16-bit types: pairwise, one packed conversion per pair)
template <class T, int V>
__device__ __forceinline__ Vec<T, V> round_vec(const float (&in)[V]) {
  Vec<T, V> t;
  if constexpr (sizeof(T) == 2 && V % 2 == 0) {
#pragma unroll
    for (int i = 0; i < V; i += 2) {
      const typename Pair16<T>::V q = from_f32x2<T>(in[i], in[i + 1]);
      t.v[i] = q[0]; t.v[i + 1] = q[1];
    }
  } else {
#pragma unroll
    for (int i = 0; i < V; ++i) t.v[i] = from_f32<T>(in[i]);
  }
  return t;
}
template <class T, int V>
__device__ __forceinline__ void store_f32(T* p, const float (&in)[V]) {
  *reinterpret_cast<Vec<T, V>*>(p) = round_vec<T, V>(in);
}

// 16 bytes held in registers between a global load and an LDS store (a plain vector type: arrays of it stay in
// registers across loop back-edges)
typedef __attribute__((ext_vector_type(4))) uint32_t Chunk;
__device__ __forceinline__ Chunk zero_chunk() { Chunk c = {0u, 0u, 0u, 0u}; return c; }

// floor(m / d) by multiplication, exact for m * d < 2^48
struct FastDiv {
  uint64_t magic; uint32_t d;
  __device__ __forceinline__ uint32_t div(uint32_t m) const { return (uint32_t)(((uint64_t)m * magic) >> 48); }
};
inline FastDiv make_fastdiv(uint32_t d) { FastDiv f; f.d = d; f.magic = (((uint64_t)1 << 48) + d - 1) / d; return f; }

// The BatchNorm affine map; the same instruction sequence in forward and backward so that the
// ReLU mask rebuilt in backward equals the one applied in forward, bit for bit.
__device__ __forceinline__ float bn_affine(float z, float scale, float shift) { return __fmaf_rn(z, scale, shift); }

inline int ceil_div(int64_t a, int64_t b) { return (int)((a + b - 1) / b); }

}  // namespace oseq
