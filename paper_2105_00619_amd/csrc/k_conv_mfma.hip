// Implicit-GEMM convolution on the matrix cores (MFMA 32x32, fp32 accumulate) for gfx950.
//
// Forward and data gradient share one kernel: out[m][n] = sum_kk A[m][kk] * B[n][kk], where
//   m  = output pixel (image, row, col),      n = output channel of this GEMM,
//   kk = (tap r, tap s, source channel) with the source channel fastest,
//   A  is gathered on the fly from the NHWC source tensor (im2col tile staged in LDS, zero outside the image),
//   B  is a [n][R*S*C_src] matrix: the (C_out,kh,kw,C_in) weights for forward, their (C_in,kh,kw,C_out)
//      transpose for the data gradient.
// Forward gathers x[n, p*stride + r - pad, q*stride + s - pad, :]; the data gradient gathers
// dz[n, (h + pad - r)/stride, (w + pad - s)/stride, :] where the division is exact.
// The weight gradient is the transposed problem (reduction over pixels) and has its own kernel.
//
// Tiling: 256 threads = 4 wavefronts of 64 lanes in a 2x2 grid; block tile 128 x BN (BN = 128 or 64), depth BK of
// 64 bytes per row (16 fp32 / 32 half elements, so one depth tile never straddles a filter tap when C_src % BK == 0).
// Each lane keeps 32 bytes of every operand row per depth tile; global loads for tile t+1 are issued before the
// MFMAs of tile t (register prefetch + two LDS buffers, one barrier per tile).
#include <algorithm>

#include "bn_fold.h"
#include "dev_common.h"
#include "epilogue.h"
#include "kernels.h"

namespace oseq {

typedef __attribute__((ext_vector_type(16))) float v16f;
typedef __attribute__((ext_vector_type(8))) __bf16 v8bf;
typedef __attribute__((ext_vector_type(8))) _Float16 v8h;
typedef __attribute__((ext_vector_type(4))) float v4f;

// 16 bytes in flight between global memory and LDS: a first-class vector value, never a stack object

enum { IG_FWD = 0, IG_DGRAD = 1 };

struct IGemmArgs {
  int srcH, srcW, srcC;   // gathered tensor
  int dstH, dstW;         // pixel grid of the result
  int M, Ng, Kg;          // GEMM sizes: rows (pixels), columns (channels), depth (R*S*srcC)
  int R, S, stride, pad, relu;
  int kt_per_split;       // depth tiles per blockIdx.z when the depth is split
  // Data gradient of a stride-2 convolution by parity classes (cls = 1): blockIdx.z is the class (ph, pw) of the
  // output pixel (h, w) = (2*hh + ph, 2*ww + pw); only the taps with (ph + pad - r) and (pw + pad - s) even reach
  // that class, so each class is its own GEMM over its tap list.  dstH / dstW are then the class grid (fullH/2,
  // fullW/2), M its pixel count, taps[c] the list (one byte per tap, r*S + s), ntaps[c] its length.
  int cls, fullH, fullW;
  int taps[4], ntaps[4];
  const uint8_t* amask;   // data gradient with an addend: ReLU bit mask the addend is multiplied by, or null
};

template <class T> struct Frag;  // 32 bytes of one operand row, and the MFMAs that consume it
template <> struct Frag<float> {
  static constexpr int BK = 16;
  v4f lo, hi;
  __device__ __forceinline__ void load(const float* p) { lo = *(const v4f*)p; hi = *(const v4f*)(p + 4); }
  __device__ __forceinline__ void load_lo(const float* p) { lo = *(const v4f*)p; }
  __device__ __forceinline__ void load_hi(const float* p) { hi = *(const v4f*)(p + 4); }
  static constexpr int HALF_STEPS = 4;  // MFMAs per operand half
  __device__ static __forceinline__ void mma_half(const Frag& a, const Frag& b, v16f& c, int half, int t) {
    c = half == 0 ? __builtin_amdgcn_mfma_f32_32x32x2f32(a.lo[t], b.lo[t], c, 0, 0, 0)
                  : __builtin_amdgcn_mfma_f32_32x32x2f32(a.hi[t], b.hi[t], c, 0, 0, 0);
  }
  static constexpr int lane_off(int g) { return g * 8; }
  static constexpr int STEPS = 8;
  __device__ static __forceinline__ void mma_step(const Frag& a, const Frag& b, v16f& c, int t) {
    c = t < 4 ? __builtin_amdgcn_mfma_f32_32x32x2f32(a.lo[t & 3], b.lo[t & 3], c, 0, 0, 0)
              : __builtin_amdgcn_mfma_f32_32x32x2f32(a.hi[t & 3], b.hi[t & 3], c, 0, 0, 0);
  }
  __device__ static __forceinline__ void mma(const Frag& a, const Frag& b, v16f& c) {
#pragma unroll
    for (int t = 0; t < 4; ++t) c = __builtin_amdgcn_mfma_f32_32x32x2f32(a.lo[t], b.lo[t], c, 0, 0, 0);
#pragma unroll
    for (int t = 0; t < 4; ++t) c = __builtin_amdgcn_mfma_f32_32x32x2f32(a.hi[t], b.hi[t], c, 0, 0, 0);
  }
};
template <> struct Frag<bf16_t> {
  static constexpr int BK = 32;
  v8bf lo, hi;
  __device__ __forceinline__ void load(const bf16_t* p) { lo = *(const v8bf*)p; hi = *(const v8bf*)(p + 8); }
  __device__ __forceinline__ void load_lo(const bf16_t* p) { lo = *(const v8bf*)p; }
  __device__ __forceinline__ void load_hi(const bf16_t* p) { hi = *(const v8bf*)(p + 8); }
  static constexpr int HALF_STEPS = 1;
  __device__ static __forceinline__ void mma_half(const Frag& a, const Frag& b, v16f& c, int half, int) {
    c = half == 0 ? __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.lo, b.lo, c, 0, 0, 0)
                  : __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.hi, b.hi, c, 0, 0, 0);
  }
  static constexpr int lane_off(int g) { return g * 16; }
  static constexpr int STEPS = 2;
  __device__ static __forceinline__ void mma_step(const Frag& a, const Frag& b, v16f& c, int t) {
    c = t == 0 ? __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.lo, b.lo, c, 0, 0, 0)
               : __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.hi, b.hi, c, 0, 0, 0);
  }
  __device__ static __forceinline__ void mma(const Frag& a, const Frag& b, v16f& c) {
    c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.lo, b.lo, c, 0, 0, 0);
    c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.hi, b.hi, c, 0, 0, 0);
  }
};
template <> struct Frag<f16_t> {
  static constexpr int BK = 32;
  v8h lo, hi;
  __device__ __forceinline__ void load(const f16_t* p) { lo = *(const v8h*)p; hi = *(const v8h*)(p + 8); }
  __device__ __forceinline__ void load_lo(const f16_t* p) { lo = *(const v8h*)p; }
  __device__ __forceinline__ void load_hi(const f16_t* p) { hi = *(const v8h*)(p + 8); }
  static constexpr int HALF_STEPS = 1;
  __device__ static __forceinline__ void mma_half(const Frag& a, const Frag& b, v16f& c, int half, int) {
    c = half == 0 ? __builtin_amdgcn_mfma_f32_32x32x16_f16(a.lo, b.lo, c, 0, 0, 0)
                  : __builtin_amdgcn_mfma_f32_32x32x16_f16(a.hi, b.hi, c, 0, 0, 0);
  }
  static constexpr int lane_off(int g) { return g * 16; }
  static constexpr int STEPS = 2;
  __device__ static __forceinline__ void mma_step(const Frag& a, const Frag& b, v16f& c, int t) {
    c = t == 0 ? __builtin_amdgcn_mfma_f32_32x32x16_f16(a.lo, b.lo, c, 0, 0, 0)
               : __builtin_amdgcn_mfma_f32_32x32x16_f16(a.hi, b.hi, c, 0, 0, 0);
  }
  __device__ static __forceinline__ void mma(const Frag& a, const Frag& b, v16f& c) {
    c = __builtin_amdgcn_mfma_f32_32x32x16_f16(a.lo, b.lo, c, 0, 0, 0);
    c = __builtin_amdgcn_mfma_f32_32x32x16_f16(a.hi, b.hi, c, 0, 0, 0);
  }
};
// Within a depth tile the two lane groups (lanes 0-31, 32-63) own disjoint halves of the depth range and every MFMA
// pairs the same depth indices of A and B, so any assignment of depth indices to (lane group, step) gives the same sum.

// SPLIT: blockIdx.z owns a fixed range of depth tiles and writes raw fp32 sums to partial[z][M][Ng]; a second
// kernel adds the ranges in order and applies the epilogue (layers with few output pixels, to fill the chip).
// Pipeline: three LDS stages, two register generations.  Iteration j: MFMAs of tile j from operand registers; the
// halves of those registers are reloaded with tile j+1 (LDS stage (j+1)%3) as soon as their MFMAs are issued; the
// global loads of tile j+3 are issued at the top and written to LDS stage j%3 at the end of iteration j+1.
template <int V> struct IC { static constexpr int value = V; };

template <class T, int BM, int BN> constexpr size_t igemm_smem_bytes() {
  constexpr size_t stages = (size_t)3 * (BM + BN) * (Frag<T>::BK + 16 / sizeof(T)) * sizeof(T);
  constexpr size_t epi = (size_t)(BM / 2) * (BN + 4) * 4;
  return stages > epi ? stages : epi;
}

template <class T, int BM, int BN, int MODE, bool SPLIT>
__global__ void __launch_bounds__(256) conv_igemm_kernel(const T* __restrict__ src, const T* __restrict__ wmat,
                                                         const float* __restrict__ bias, const T* __restrict__ addend,
                                                         T* __restrict__ out, float* __restrict__ partial,
                                                         float* __restrict__ stat_partial, IGemmArgs a) {
  constexpr int BK = Frag<T>::BK;
  constexpr int EV = 16 / (int)sizeof(T);   // elements per 16-byte chunk
  constexpr int PITCH = BK + EV;            // LDS row pitch in elements (80 bytes)
  constexpr int MI = BM / 64, NI = BN / 64; // 32x32 MFMA tiles per wavefront
  constexpr int A_CH = BM * 4 / 256;        // 16-byte chunks per thread and depth tile (4 chunks per row)
  constexpr int B_CH = BN * 4 / 256;
  constexpr int STAGE = (BM + BN) * PITCH;  // elements per LDS stage: A rows then B rows
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  T* lds = reinterpret_cast<T*>(smem_raw);

  // kernel arguments used inside the loaders, as plain scalars
  const int srcH = a.srcH, srcW = a.srcW, srcC = a.srcC, S_ = a.S, stride = a.stride, pad = a.pad;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1, g = lane >> 5, l32 = lane & 31;
  const int m0 = blockIdx.x * BM, n0 = blockIdx.y * BN;
  const int vec = tid & 3, row0 = tid >> 2;  // this thread's chunk column and first row

  // pixel coordinates of this thread's A rows
  const int cz = a.cls ? blockIdx.z : 0;              // parity class
  const int cph = cz >> 1, cpw = cz & 1;
  const int ctaps = a.cls ? a.taps[cz] : 0;
  int pn[A_CH], pa[A_CH], pb[A_CH];
#pragma unroll
  for (int i = 0; i < A_CH; ++i) {
    const int m = m0 + row0 + i * 64;
    const int mm = m < a.M ? m : 0;
    pb[i] = mm % a.dstW;
    const int t = mm / a.dstW;
    pa[i] = t % a.dstH;
    pn[i] = m < a.M ? t / a.dstH : -1;  // -1: row beyond the last pixel
    if (a.cls) { pa[i] = 2 * pa[i] + cph; pb[i] = 2 * pb[i] + cpw; }
  }
  const T* brow[B_CH];
#pragma unroll
  for (int i = 0; i < B_CH; ++i) brow[i] = wmat + (int64_t)(n0 + row0 + i * 64) * (a.R * a.S * srcC) + vec * EV;

  // Global loads are unconditional (addresses of out-of-image taps are clamped into the tensor) and the zeroing is
  // applied when the chunk is written to LDS: straight-line loads let the hardware keep several generations in flight.
  Chunk ra[2][A_CH], rb[2][B_CH];
  unsigned okm[2] = {0u, 0u};  // per generation: bit i set if A chunk i is inside the image
  auto gload = [&, srcH, srcW, srcC, S_, stride, pad](auto P, int kt) {
    constexpr int p = decltype(P)::value;
    const int kk0 = kt * BK;
    const int tapi = kk0 / srcC, c0 = kk0 - tapi * srcC;
    const int tap = a.cls ? (ctaps >> (8 * tapi)) & 0xff : tapi;  // filter tap r*S + s of this depth tile
    const int r = tap / S_, s = tap - r * S_;
    const int kkw = tap * srcC + c0;                              // its depth offset in the weight rows
    unsigned m = 0u;
#pragma unroll
    for (int i = 0; i < A_CH; ++i) {
      int y, x;
      bool ok = pn[i] >= 0;
      if (MODE == IG_FWD) {
        y = pa[i] * stride + r - pad;
        x = pb[i] * stride + s - pad;
      } else {
        const int ty = pa[i] + pad - r, tx = pb[i] + pad - s;
        ok = ok && ty >= 0 && tx >= 0;
        if (stride == 2) { ok = ok && !((ty | tx) & 1); y = ty >> 1; x = tx >> 1; } else { y = ty; x = tx; }
      }
      ok = ok && y >= 0 && y < srcH && x >= 0 && x < srcW;
      const int yc = ok ? y : 0, xc = ok ? x : 0, nc = ok ? pn[i] : 0;
      ra[p][i] = *reinterpret_cast<const Chunk*>(src + (((int64_t)nc * srcH + yc) * srcW + xc) * srcC + c0 + vec * EV);
      m |= ok ? (1u << i) : 0u;
    }
    okm[p] = m;
#pragma unroll
    for (int i = 0; i < B_CH; ++i) rb[p][i] = *reinterpret_cast<const Chunk*>(brow[i] + kkw);
  };
  auto sstore = [&](auto P, int stage) {  // register generation p -> LDS stage
    constexpr int p = decltype(P)::value;
    T* st = lds + stage * STAGE;
#pragma unroll
    for (int i = 0; i < A_CH; ++i)
      *reinterpret_cast<Chunk*>(&st[(row0 + i * 64) * PITCH + vec * EV]) = ((okm[p] >> i) & 1u) ? ra[p][i] : zero_chunk();
#pragma unroll
    for (int i = 0; i < B_CH; ++i) *reinterpret_cast<Chunk*>(&st[(BM + row0 + i * 64) * PITCH + vec * EV]) = rb[p][i];
  };

  v16f acc[MI][NI];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NI; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  const int kt0 = SPLIT ? blockIdx.z * a.kt_per_split : 0;
  const int nkt = (a.cls ? a.ntaps[cz] * srcC : a.Kg) / BK;  // depth tiles of this GEMM
  const int kt1 = SPLIT ? (kt0 + a.kt_per_split < nkt ? kt0 + a.kt_per_split : nkt) : nkt;
  const int n = kt1 > kt0 ? kt1 - kt0 : 0;
  // prologue: tiles 0 and 1 into LDS stages 0 and 1, tile 2 on its way in generation 0
  if (n > 0) { gload(IC<0>{}, kt0); sstore(IC<0>{}, 0); }
  if (n > 1) { gload(IC<1>{}, kt0 + 1); sstore(IC<1>{}, 1); }
  if (n > 2) gload(IC<0>{}, kt0 + 2);
  __syncthreads();
  const int afrag = (wm * (BM / 2) + l32) * PITCH + Frag<T>::lane_off(g);
  const int bfrag = (BM + wn * (BN / 2) + l32) * PITCH + Frag<T>::lane_off(g);
  Frag<T> fa[MI], fb[NI];
  if (n > 0) {
#pragma unroll
    for (int i = 0; i < MI; ++i) fa[i].load(lds + afrag + i * 32 * PITCH);
#pragma unroll
    for (int jn = 0; jn < NI; ++jn) fb[jn].load(lds + bfrag + jn * 32 * PITCH);
  }
  // iteration j: generation (j & 1) holds tile j+2 (issued at iteration j-1 or in the prologue)
  // TAIL = 0: steady state, every step unconditional (a branch around the loads would make the compiler wait for
  // the newest loads before each LDS store); TAIL = 1: the last iterations, with the range checks.
  auto body = [&](auto P, auto TAILC, int j, int stage) {
    constexpr int p = decltype(P)::value;  // = j & 1
    constexpr bool TAIL = decltype(TAILC)::value != 0;
    const T* nxt = lds + (stage == 2 ? 0 : stage + 1) * STAGE;
    const bool has_next = TAIL ? j + 1 < n : true;
    if (!TAIL || j + 3 < n) gload(IC<1 - p>{}, kt0 + j + 3);
#pragma unroll
    for (int st = 0; st < Frag<T>::HALF_STEPS; ++st)
#pragma unroll
      for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int jn = 0; jn < NI; ++jn) Frag<T>::mma_half(fa[i], fb[jn], acc[i][jn], 0, st);
    __builtin_amdgcn_sched_barrier(0);
    if (has_next) {
#pragma unroll
      for (int i = 0; i < MI; ++i) fa[i].load_lo(nxt + afrag + i * 32 * PITCH);
#pragma unroll
      for (int jn = 0; jn < NI; ++jn) fb[jn].load_lo(nxt + bfrag + jn * 32 * PITCH);
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int st = 0; st < Frag<T>::HALF_STEPS; ++st)
#pragma unroll
      for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int jn = 0; jn < NI; ++jn) Frag<T>::mma_half(fa[i], fb[jn], acc[i][jn], 1, st);
    __builtin_amdgcn_sched_barrier(0);
    if (has_next) {
#pragma unroll
      for (int i = 0; i < MI; ++i) fa[i].load_hi(nxt + afrag + i * 32 * PITCH);
#pragma unroll
      for (int jn = 0; jn < NI; ++jn) fb[jn].load_hi(nxt + bfrag + jn * 32 * PITCH);
    }
    if (!TAIL || j + 2 < n) sstore(P, stage == 0 ? 2 : stage - 1);  // tile j+2 -> stage (j+2)%3
    __syncthreads();
  };
  {
    int stage = 0, j = 0;
    for (; j + 4 < n; j += 2) {
      body(IC<0>{}, IC<0>{}, j, stage);
      stage = stage == 2 ? 0 : stage + 1;
      body(IC<1>{}, IC<0>{}, j + 1, stage);
      stage = stage == 2 ? 0 : stage + 1;
    }
    for (; j < n; j += 2) {
      body(IC<0>{}, IC<1>{}, j, stage);
      stage = stage == 2 ? 0 : stage + 1;
      if (j + 1 < n) {
        body(IC<1>{}, IC<1>{}, j + 1, stage);
        stage = stage == 2 ? 0 : stage + 1;
      }
    }
  }

  // epilogue through LDS, one half of the rows (the two wavefronts with the same wm) at a time, as fp32 [row][BN+4];
  // the store half (bias / addend / ReLU, rounding, stores, BatchNorm sums) is shared with the other kernels
  {
    float* ep = reinterpret_cast<float*>(smem_raw);
    constexpr int EP_PITCH = BN + 4;
    constexpr int HR = BM / 2;  // rows per pass
    constexpr bool STAT = MODE == IG_FWD && !SPLIT;
    float ss[8], qq[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) { ss[k] = 0.f; qq[k] = 0.f; }
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      __syncthreads();
      if (wm == u) {
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
          for (int jn = 0; jn < NI; ++jn)
#pragma unroll
            for (int e = 0; e < 16; ++e)
              ep[(i * 32 + 8 * (e >> 2) + 4 * g + (e & 3)) * EP_PITCH + wn * (BN / 2) + jn * 32 + l32] = acc[i][jn][e];
      }
      __syncthreads();
      auto rowoff = [&](int row) -> int64_t {
        const int grow = m0 + u * HR + row;
        if (grow >= a.M) return -1;
        int64_t opix = grow;
        if (a.cls) {  // class-local pixel -> pixel of the full grid
          const int ww = grow % a.dstW, t2 = grow / a.dstW;
          const int hh = t2 % a.dstH, nn = t2 / a.dstH;
          opix = ((int64_t)nn * a.fullH + 2 * hh + cph) * a.fullW + 2 * ww + cpw;
        }
        return opix * a.Ng;
      };
      if (SPLIT) {
        epi_store_partial<BN, HR>(ep, tid, n0, partial + (int64_t)blockIdx.z * a.M * a.Ng, rowoff);
      } else if (STAT && stat_partial) {
        epi_store_pass<T, BN, HR, MODE == IG_FWD, MODE == IG_DGRAD, true>(ep, tid, n0, bias, addend, a.amask, out, a.relu, rowoff, ss, qq);
      } else {
        epi_store_pass<T, BN, HR, MODE == IG_FWD, MODE == IG_DGRAD, false>(ep, tid, n0, bias, addend, a.amask, out, a.relu, rowoff, ss, qq);
      }
    }
    if (STAT && stat_partial)
      epi_stat_combine<BN>(ep, tid, ss, qq, stat_partial + ((int64_t)blockIdx.x * 2 + 0) * a.Ng + n0,
                           stat_partial + ((int64_t)blockIdx.x * 2 + 1) * a.Ng + n0);
  }
}

// ------------------------------------------------------------------------------------------------------------
// 3x3, stride 1: the input patch of the block's pixels (with its halo and zero border) is staged in LDS once per
// channel chunk and serves all nine filter taps, so the vector-memory path carries every input line once instead
// of nine times; only the 64-byte-deep weight tile changes from tap to tap.
//   block = 256 threads = 4 wavefronts (2 x 2); block tile = 64*MI pixel rows x BN channels; a wavefront owns 32*MI
//   rows and BN/2 channels: MI x (BN/64) MFMA 32x32 tiles.  The rows are SUBT pixel sub-tiles of 64*MI/SUBT pixels
//   (TI images x TR rows x TC columns each, with their own halo).  Instantiated: (MI 2, SUBT 1) with 128 or 64
//   channels and (1, 1) with 64; two blocks share a CU, three with 64 channels (registers capped, patch
//   buffers sized for the layer's tile).
//   LDS: 2 patch buffers [SUBT*256 positions][80 B], 3 weight stages [BN][80 B], address tables.
//   Pipeline (one barrier per tap): the weight tile of (chunk c+1, tap t) is requested before the MFMAs of (c, t)
//   and parked in registers until the end of step (c+1, t-1); the next chunk's patch is requested during taps 0-3
//   and stored during taps 4-7.  All loads are straight-line, so several steps of loads stay in flight.
//   The data gradient of a stride-1 convolution is the same computation on dz with the taps visited in reverse and
//   the border (kh-1-pad).
// ------------------------------------------------------------------------------------------------------------
struct PatchArgs {
  int N, srcH, srcW, srcC;   // gathered tensor
  int dstH, dstW, Ng;        // pixel grid and channels of the result
  int pad, flip;             // border of the gather; flip: weight tap index 8 - t (data gradient)
  int TI, TR, TC, SR, SC, NPOS, TP;
  int tiles_r, tiles_c, NT;
  int relu;
  int chunks_per_split;      // channel chunks per blockIdx.z (all of them when the depth is not split)
  int row_pitch;             // bytes between staged patch rows in LDS (>= SC * 80, padded against bank conflicts)
  int patch_elems;           // elements of one staged patch buffer (its rows times row_pitch, rounded up to 16 bytes)
  int xcd_group;             // 1: blocks are renumbered so that the row tiles of one weight slice run on one XCD;
                             // 2: so that the channel blocks and depth ranges of one row tile do (row_blocks: row tiles)
  int row_blocks;
  const uint8_t* amask;      // data gradient with an addend: ReLU bit mask the addend is multiplied by, or null
  const float* fold;         // FOLD (forward): src is the z of a BatchNorm + ReLU, this its [4][srcC] statistics tensor; the
                             // pieces of the patch become the activation (scale, shift, ReLU, one rounding) on their way
                             // to LDS; positions outside the image stay zero
};

constexpr int PATCH_MAX_POS = 256;  // positions per sub-tile

template <class T, int BN, int MI, int SUBT, bool STAT, bool FOLD = false>
__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(BN == 64 ? 3 : 1, BN == 64 ? 3 : 2)))
conv3x3_patch_kernel(const T* __restrict__ src, const T* __restrict__ wmat, const float* __restrict__ bias,
                     const T* __restrict__ addend, T* __restrict__ out, float* __restrict__ partial,
                     float* __restrict__ stat_partial, PatchArgs a) {
  constexpr int ROWS = 64 * MI;              // pixel rows of the block
  constexpr int TPC = ROWS / SUBT;           // rows (pixel capacity) per sub-tile
  constexpr int NSLOT = 4 * SUBT;            // 16-byte patch pieces per thread and channel chunk
  constexpr int SPT = NSLOT / 4;             // pieces requested / stored per tap
  constexpr int CCE = Frag<T>::BK;           // channels per chunk (64 bytes)
  constexpr int EV = 16 / (int)sizeof(T);
  constexpr int PITCH = CCE + EV;            // elements per LDS row (80 bytes)
  constexpr int NI = BN / 64;
  constexpr int B_CH = BN * 4 / 256;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  const int PBUF = a.patch_elems;                                             // one patch buffer, sized for this layer
  T* patch = reinterpret_cast<T*>(smem_raw);                                  // [2][PBUF]
  T* Bs = patch + 2 * PBUF;                                                   // [3][BN][PITCH]
  int64_t* src_off = reinterpret_cast<int64_t*>(Bs + 3 * BN * PITCH);         // [SUBT*PATCH_MAX_POS]
  int64_t* out_off = src_off + SUBT * PATCH_MAX_POS;                          // [256]
  int* apos = reinterpret_cast<int*>(out_off + 256);                          // [256]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1, g = lane >> 5, l32 = lane & 31;
  // Block coordinates: (row tile, channel block, depth range).  Workgroups go to the 8 XCDs round-robin by their
  // linear index, and every XCD has an L2 of its own.  With large weights and few pixels the row tiles of one
  // (channel block, depth range) all read the same weight slice: renumbered, they run on one XCD, which then fetches
  // the slice once instead of all eight doing so.  Needs (channel blocks x depth ranges) % 8 == 0 (launcher).
  int bx = blockIdx.x, by = blockIdx.y, bz = blockIdx.z;
  if (a.xcd_group == 1) {
    const unsigned lin = blockIdx.x + gridDim.x * (blockIdx.y + gridDim.y * blockIdx.z);
    const unsigned xcd = lin & 7u, slot = lin >> 3;
    const unsigned grp = (slot / gridDim.x) * 8u + xcd;  // index of the (channel block, depth range) pair
    bx = (int)(slot % gridDim.x); by = (int)(grp % gridDim.y); bz = (int)(grp / gridDim.y);
  }
  // Many pixels and two or more channel blocks: the blocks of one row tile all stage the same patches of the source;
  // renumbered onto one XCD in consecutive slots they fetch them from HBM once (256 -> 256 channels at 262 144 pixels,
  // bf16: 293 MB per launch without it for 135 MB of operands).  The grid's x extent is then the number of row tiles
  // rounded up to a multiple of 8.
  if (a.xcd_group == 2) {
    const unsigned lin = blockIdx.x + gridDim.x * (blockIdx.y + gridDim.y * blockIdx.z);
    const unsigned xcd = lin & 7u, slot = lin >> 3;
    const unsigned per = gridDim.y * gridDim.z, idx = slot % per;
    bx = (int)((slot / per) * 8u + xcd); by = (int)(idx % gridDim.y); bz = (int)(idx / gridDim.y);
    if (bx >= a.row_blocks) return;
  }
  const int n0c = by * BN;
  const int npos2 = SUBT * a.NPOS;
  const int srcC = a.srcC, flip = a.flip, SC = a.SC;
  const int RPE = a.row_pitch / (int)sizeof(T);  // elements between staged patch rows

  // ---- address tables ------------------------------------------------------------------------------------------
  for (int e = tid; e < npos2; e += 256) {
    const int u = e / a.NPOS, rem = e - u * a.NPOS;
    const int ti = rem / (a.SR * a.SC), rr = rem - ti * (a.SR * a.SC);
    const int sy = rr / a.SC, sx = rr - sy * a.SC;
    const int tile = SUBT * bx + u;
    int64_t off = -1;
    if (tile < a.NT) {
      const int ci = tile % a.tiles_c, t2 = tile / a.tiles_c;
      const int ri = t2 % a.tiles_r, ii = t2 / a.tiles_r;
      const int n = ii * a.TI + ti, y = ri * a.TR - a.pad + sy, x = ci * a.TC - a.pad + sx;
      if (n < a.N && y >= 0 && y < a.srcH && x >= 0 && x < a.srcW) off = (((int64_t)n * a.srcH + y) * a.srcW + x) * a.srcC;
    }
    src_off[e] = off;
  }
  {
    const int m2 = tid, u = m2 / TPC, m = m2 - u * TPC;
    const int tile = SUBT * bx + u;
    int64_t off = -1;
    int ap = 0;
    if (m2 < ROWS && m < a.TP && tile < a.NT) {
      const int ti = m / (a.TR * a.TC), rr = m - ti * (a.TR * a.TC);
      const int tr = rr / a.TC, tc = rr - tr * a.TC;
      const int ci = tile % a.tiles_c, t2 = tile / a.tiles_c;
      const int ri = t2 % a.tiles_r, ii = t2 / a.tiles_r;
      const int n = ii * a.TI + ti, p = ri * a.TR + tr, q = ci * a.TC + tc;
      ap = ((u * a.TI + ti) * a.SR + tr) * RPE + tc * PITCH;  // LDS element offset of tap (0,0)
      if (n < a.N && p < a.dstH && q < a.dstW) off = (((int64_t)n * a.dstH + p) * a.dstW + q) * a.Ng;
    }
    out_off[m2] = off;
    apos[m2] = ap;
  }
  __syncthreads();

  // channel chunks of this block: all of them, or the range of blockIdx.z (raw sums go to `partial`, a second
  // kernel adds the ranges in order and applies the epilogue)
  const int cb = bz * a.chunks_per_split;
  const int ce = cb + a.chunks_per_split < srcC / CCE ? cb + a.chunks_per_split : srcC / CCE;
  const int Kg = 9 * srcC;

  // ---- loaders ---------------------------------------------------------------------------------------------------
  Chunk PR[NSLOT];  // patch chunks in flight (next channel chunk)
  // weight tiles in flight: one generation per tap, requested a whole channel chunk (nine steps) ahead
  // (a = rows 0-63, b = rows 64-127 of the tile)
  Chunk BRa[9], BRb[9];
  const int bvec = tid & 3, brow0 = tid >> 2;
  // patch pieces of this thread: slot sl covers the 16-byte piece idx = sl*256 + tid.  Loads are unconditional
  // (pieces outside the image read the tensor's first pixel) and are zeroed when written to LDS.
  const T* pptr[NSLOT];
  int pdst[NSLOT];  // LDS element offset of the piece within a patch buffer
  unsigned pvalid = 0u, pstore = 0u;
#pragma unroll
  for (int sl = 0; sl < NSLOT; ++sl) {
    const int idx = sl * 256 + tid;
    const int pos = idx >> 2, v = idx & 3;
    int64_t off = 0;
    int dst = 0;
    if (pos < npos2) {
      pstore |= 1u << sl;
      const int64_t o = src_off[pos];
      if (o >= 0) { off = o; pvalid |= 1u << sl; }
      const int prow = pos / SC;
      dst = prow * RPE + (pos - prow * SC) * PITCH + v * EV;
    }
    pptr[sl] = src + off + v * EV;
    pdst[sl] = dst;
  }
  auto patch_load = [&](int slot, int chunk) { return *reinterpret_cast<const Chunk*>(pptr[slot] + chunk * CCE); };
  // FOLD: all pieces of a thread cover channels [(tid & 3) * EV, + EV) of the chunk; their scale and shift are
  // requested with the first pieces of a chunk and used when the pieces are stored
  float fsc[EV], fsh[EV];
  auto fold_load = [&](int chunk) {
    if (FOLD) {
      const int c = chunk * CCE + (tid & 3) * EV;
      load_f32<float, EV>(a.fold + 2 * srcC + c, fsc);
      load_f32<float, EV>(a.fold + 3 * srcC + c, fsh);
    }
  };
  auto patch_store = [&](int slot, int buf, const Chunk& c) {
    if ((pstore >> slot) & 1u) {
      Chunk v = c;
      if (FOLD) v = bn_fold_chunk<T>(c, fsc, fsh);
      *reinterpret_cast<Chunk*>(&patch[buf * PBUF + pdst[slot]]) = ((pvalid >> slot) & 1u) ? v : zero_chunk();
    }
  };
  const T* wrow = wmat + (int64_t)(n0c + brow0) * Kg + bvec * EV;
  // weight tile of global step gs = chunk*9 + tap -> registers REG
  // weight tile of tap slot t_ of channel chunk ch_ -> registers of generation t_
#define B_LOAD(t_, ch_)                                                                                       \
  {                                                                                                           \
    const int tap_ = flip ? 8 - (t_) : (t_);                                                                  \
    const T* wp_ = wrow + tap_ * srcC + (ch_) * CCE;                                                          \
    BRa[t_] = *reinterpret_cast<const Chunk*>(wp_);                                                           \
    if (B_CH > 1) BRb[t_] = *reinterpret_cast<const Chunk*>(wp_ + (int64_t)64 * Kg);                          \
  }
#define B_STORE(t_, stage_)                                                                                   \
  {                                                                                                           \
    *reinterpret_cast<Chunk*>(&Bs[((stage_) * BN + brow0) * PITCH + bvec * EV]) = BRa[t_];                    \
    if (B_CH > 1) *reinterpret_cast<Chunk*>(&Bs[((stage_) * BN + brow0 + 64) * PITCH + bvec * EV]) = BRb[t_]; \
  }

  // ---- prologue -----------------------------------------------------------------------------------------------
#pragma unroll
  for (int sl = 0; sl < NSLOT; ++sl) PR[sl] = patch_load(sl, cb);
  fold_load(cb);
#pragma unroll
  for (int t = 0; t < 9; ++t) B_LOAD(t, cb);
#pragma unroll
  for (int sl = 0; sl < NSLOT; ++sl) patch_store(sl, 0, PR[sl]);
  B_STORE(0, 0);
  B_STORE(1, 1);
  __syncthreads();

  int arow[MI];  // LDS element offset of tap (0,0) for this lane's 32-row groups
#pragma unroll
  for (int i = 0; i < MI; ++i) arow[i] = apos[wm * (32 * MI) + i * 32 + l32] + Frag<T>::lane_off(g);
  const int bfrag = (wn * (BN / 2) + l32) * PITCH + Frag<T>::lane_off(g);  // this lane's row in a weight stage

  v16f acc[MI][NI];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NI; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  // Operand fragments live in one set of registers.  Each half (first / second 16 bytes of the 32-byte depth slice) is
  // reloaded for the next step right after the MFMAs that consumed it have been issued, so the LDS reads of step g+1
  // run under the MFMAs of step g and nothing waits on LDS latency.  Weight stage = step % 3; the weight tile of step
  // g+2 is written at the end of step g, the next chunk's patch during taps 4-7, so both are complete one barrier
  // before their first read.
  Frag<T> fa[MI], fb[NI];
#pragma unroll
  for (int i = 0; i < MI; ++i) fa[i].load(patch + arow[i]);
#pragma unroll
  for (int j = 0; j < NI; ++j) fb[j].load(&Bs[bfrag + j * 32 * PITCH]);

  // one channel chunk = nine taps; LAST = no chunk follows (no patch prefetch, weight requests stop at the end)
  auto chunk_body = [&](auto LAST, int chunk) {
    constexpr bool last = decltype(LAST)::value != 0;
    const int pbuf = (chunk - cb) & 1;
    const T* pcur = patch + pbuf * PBUF;
    const T* pnxt = patch + (pbuf ^ 1) * PBUF;
#pragma unroll
    for (int t = 0; t < 9; ++t) {
      // where the next step reads its operands
      const bool has_next = !last || t + 1 < 9;
      const int tn = (t + 1) % 9;
      const T* pn = t + 1 < 9 ? pcur : pnxt;
      const int tapoff_n = (tn / 3) * RPE + (tn % 3) * PITCH;
      const T* bn_ = &Bs[((t + 1) % 3) * BN * PITCH + bfrag];
      // requests: the weight tile this tap will need in the next chunk, two pieces of the next patch during taps 0-3
      if (!last) B_LOAD(t, chunk + 1);
      if (!last && t < 4) {
#pragma unroll
        for (int q = 0; q < SPT; ++q) PR[SPT * t + q] = patch_load(SPT * t + q, chunk + 1);
        if (t == 0) fold_load(chunk + 1);
      }
      // first halves
#pragma unroll
      for (int st = 0; st < Frag<T>::HALF_STEPS; ++st)
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
          for (int j = 0; j < NI; ++j) Frag<T>::mma_half(fa[i], fb[j], acc[i][j], 0, st);
      __builtin_amdgcn_sched_barrier(0);
      if (has_next) {
#pragma unroll
        for (int i = 0; i < MI; ++i) fa[i].load_lo(pn + arow[i] + tapoff_n);
#pragma unroll
        for (int j = 0; j < NI; ++j) fb[j].load_lo(bn_ + j * 32 * PITCH);
      }
      __builtin_amdgcn_sched_barrier(0);
      // second halves
#pragma unroll
      for (int st = 0; st < Frag<T>::HALF_STEPS; ++st)
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
          for (int j = 0; j < NI; ++j) Frag<T>::mma_half(fa[i], fb[j], acc[i][j], 1, st);
      __builtin_amdgcn_sched_barrier(0);
      if (has_next) {
#pragma unroll
        for (int i = 0; i < MI; ++i) fa[i].load_hi(pn + arow[i] + tapoff_n);
#pragma unroll
        for (int j = 0; j < NI; ++j) fb[j].load_hi(bn_ + j * 32 * PITCH);
      }
      // parked data goes to LDS: weight tile of step g+2, patch pieces requested four taps ago
      if (t + 2 < 9) B_STORE(t + 2, (t + 2) % 3) else if (!last) B_STORE(t + 2 - 9, (t + 2) % 3)
      if (!last && t >= 4 && t < 8) {
#pragma unroll
        for (int q = 0; q < SPT; ++q) patch_store(SPT * (t - 4) + q, pbuf ^ 1, PR[SPT * (t - 4) + q]);
      }
      __syncthreads();
    }
  };
  for (int chunk = cb; chunk + 1 < ce; ++chunk) chunk_body(IC<0>{}, chunk);
  chunk_body(IC<1>{}, ce - 1);

  // ---- epilogue ---------------------------------------------------------------------------------------------------
  // The accumulators go through LDS (the patch buffers are free now), the rows of one wavefront pair at a time, as
  // fp32 [row][BN + 4]; the store half (bias / addend / ReLU, rounding, stores of whole rows, BatchNorm sums of the
  // stored values) is shared with the other kernels.
  {
    float* ep = reinterpret_cast<float*>(smem_raw);
    constexpr int EP_PITCH = BN + 4;
    constexpr int HR = 32 * MI;  // rows per pass
    float ss[8], qq[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) { ss[k] = 0.f; qq[k] = 0.f; }
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      __syncthreads();
      if (wm == u) {
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
          for (int j = 0; j < NI; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e)
              ep[(i * 32 + 8 * (e >> 2) + 4 * g + (e & 3)) * EP_PITCH + wn * (BN / 2) + j * 32 + l32] = acc[i][j][e];
      }
      __syncthreads();
      auto rowoff = [&](int row) -> int64_t { return out_off[u * HR + row]; };
      if (partial)
        epi_store_partial<BN, HR>(ep, tid, n0c, partial + (int64_t)bz * ((int64_t)a.N * a.dstH * a.dstW * a.Ng), rowoff);
      else
        epi_store_pass<T, BN, HR, true, !STAT, STAT>(ep, tid, n0c, bias, addend, a.amask, out, a.relu, rowoff, ss, qq);
    }
    if (STAT)
      epi_stat_combine<BN>(ep, tid, ss, qq, stat_partial + ((int64_t)bx * 2 + 0) * a.Ng + n0c,
                           stat_partial + ((int64_t)bx * 2 + 1) * a.Ng + n0c);
  }
}

#undef B_LOAD
#undef B_STORE

// Sum of the depth ranges in order, then bias / residual addend / ReLU, one rounding, store.  A block covers 64 rows
// x 64 channels (thread = 4 channels of every 16th row), so that it can also produce the per-channel sums of the
// stored values for the BatchNorm that follows: stat_partial [ceil(M / 64)][2][Ng], or null.
constexpr int SPLIT_EPI_ROWS = 64;
template <class T>
__global__ void __launch_bounds__(256) splitk_epilogue_kernel(const float* __restrict__ partial, int splits, int64_t M, int Ng,
                                                              const float* __restrict__ bias, const T* __restrict__ addend,
                                                              const uint8_t* __restrict__ amask, T* __restrict__ out,
                                                              float* __restrict__ stat_partial, int relu) {
  __shared__ float red[2][16][64];
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  const int col = blockIdx.y * 64 + tx * 4;
  const int64_t n = M * Ng;
  float bv[4] = {0.f, 0.f, 0.f, 0.f};
  if (bias) {
#pragma unroll
    for (int e = 0; e < 4; ++e) bv[e] = bias[col + e];
  }
  float ss[4] = {0.f, 0.f, 0.f, 0.f}, qq[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int it = 0; it < SPLIT_EPI_ROWS / 16; ++it) {
    const int64_t row = (int64_t)blockIdx.x * SPLIT_EPI_ROWS + it * 16 + ty;
    if (row < M) {
      const int64_t i = row * Ng + col;
      v4f acc = *reinterpret_cast<const v4f*>(partial + i);
      for (int z = 1; z < splits; ++z) acc += *reinterpret_cast<const v4f*>(partial + (int64_t)z * n + i);
      float r[4];
      // the addend's ReLU bits, if it has any: four consecutive elements lie in one byte (i is a multiple of 4)
      unsigned mb = 0xfu;
      if (addend && amask) mb = sizeof(T) == 2 ? (amask[i >> 3] >> (i & 4)) & 15u : amask[i >> 2] & 15u;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        float v = acc[e] + bv[e];
        if (addend && ((mb >> e) & 1u)) v += to_f32(addend[i + e]);
        r[e] = relu ? fmaxf(v, 0.f) : v;
      }
      store_f32<T, 4>(out + i, r);
      if (stat_partial) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float v = to_f32(from_f32<T>(r[e]));  // as stored
          ss[e] += v; qq[e] = __fmaf_rn(v, v, qq[e]);
        }
      }
    }
  }
  if (stat_partial) {  // the 16 row groups of a channel, added in a fixed order
#pragma unroll
    for (int e = 0; e < 4; ++e) { red[0][ty][tx * 4 + e] = ss[e]; red[1][ty][tx * 4 + e] = qq[e]; }
    __syncthreads();
    if (threadIdx.x < 128) {
      const int which = threadIdx.x >> 6, c = threadIdx.x & 63;
      float t = 0.f;
#pragma unroll
      for (int y = 0; y < 16; ++y) t += red[which][y][c];
      stat_partial[((int64_t)blockIdx.x * 2 + which) * Ng + blockIdx.y * 64 + c] = t;
    }
  }
}

template <class T>
static void launch_splitk_epilogue(hipStream_t st, const float* partial, int splits, int64_t M, int Ng, const float* bias,
                                   const void* addend, const uint8_t* amask, void* out, float* stat_partial, int relu) {
  dim3 grid(ceil_div(M, SPLIT_EPI_ROWS), Ng / 64);  // Ng % 64 == 0 for every MFMA convolution
  OSEQ_LAUNCH(splitk_epilogue_kernel<T>, grid, dim3(256), 0, st, partial, splits, M, Ng, bias, (const T*)addend, amask,
                     (T*)out, stat_partial, relu);
}

// LDS of the patch kernel: two patch buffers of patch_elems elements, three weight stages, the address tables
template <class T> constexpr size_t patch_smem_bytes(int bn, int subt, int64_t patch_elems) {
  return (size_t)(2 * patch_elems + 3 * bn * (Frag<T>::BK + 16 / sizeof(T))) * sizeof(T) + subt * PATCH_MAX_POS * 8 +
         256 * 8 + 256 * 4;
}
template <class T> constexpr size_t patch_smem_max(int bn, int subt) {
  return patch_smem_bytes<T>(bn, subt, (int64_t)subt * PATCH_MAX_POS * (Frag<T>::BK + 16 / sizeof(T)));
}

// tile geometry of the patch kernel for a (dstH x dstW) pixel grid gathered with a 3x3 window and sub-tiles of up to
// `cap` pixels; false if it does not fit
static bool patch_geometry(int N, int dstH, int dstW, int cap, PatchArgs& a) {
  int tc = dstW < cap ? dstW : cap;
  int tr = cap / tc; if (tr > dstH) tr = dstH; if (tr < 1) tr = 1;
  int ti = (tr == dstH && tc == dstW) ? cap / (dstH * dstW) : 1;
  if (ti > N) ti = N; if (ti < 1) ti = 1;
  while (ti > 1 && ti * (tr + 2) * (tc + 2) > PATCH_MAX_POS) ti /= 2;
  while (tr > 1 && ti * (tr + 2) * (tc + 2) > PATCH_MAX_POS) --tr;
  while (tc > 1 && ti * (tr + 2) * (tc + 2) > PATCH_MAX_POS) tc /= 2;
  if (ti * (tr + 2) * (tc + 2) > PATCH_MAX_POS) return false;
  a.TI = ti; a.TR = tr; a.TC = tc; a.SR = tr + 2; a.SC = tc + 2;
  a.NPOS = ti * a.SR * a.SC; a.TP = ti * tr * tc;
  a.tiles_r = (dstH + tr - 1) / tr; a.tiles_c = (dstW + tc - 1) / tc;
  a.NT = ((N + ti - 1) / ti) * a.tiles_r * a.tiles_c;
  return true;
}

// Bytes between staged patch rows.  A lane group reads 16 bytes per lane at consecutive pixels: within a row of TC
// pixels the 80-byte position pitch spreads them over the LDS banks, and the row pitch is padded so that the next
// rows of the tile land on the banks the previous ones left free (TC = 8: 128 mod 256, TC = 4: 64, TC = 2: 32);
// kept at SC * 80 when the padded rows would not fit the patch buffer.
static constexpr int g_patch_pad_rows = 1;  // compile-time switch
static int patch_row_pitch(const PatchArgs& a, int subt) {
  const int base = a.SC * 80;
  int want = -1;
  if (a.TC == 8) want = 128; else if (a.TC == 4) want = 64; else if (a.TC == 2) want = 32;
  if (want < 0 || !g_patch_pad_rows) return base;
  int rp = base / 256 * 256 + want;
  if (rp < base) rp += 256;
  const int64_t rows = (int64_t)subt * a.TI * a.SR;
  return rows * rp <= (int64_t)subt * PATCH_MAX_POS * 80 ? rp : base;
}

// Block shapes of the patch kernel, largest first: {MI, SUBT, widest BN}.  The first one that gives the chip
// `g_patch_fill` blocks is taken, else the one with the most blocks if that reaches `g_patch_min_blocks`
// (shape-only rule, so the choice is the same on every run).
struct PatchShape { int mi, subt, bn, splits; };
static constexpr int g_patch_min_blocks = 64;   // compile-time constants
static constexpr int g_patch_fill = 512;
static constexpr int g_patch_shapes = 0x7;      // bit i: candidate i allowed
static constexpr int g_patch_split = 1;         // allow the depth split
static constexpr int g_patch_halo2 = 9;         // largest staged positions : pixels ratio, times two
static constexpr int g_patch_target_small = 512;  // blocks aimed at by the depth split for the smallest block shape in fp32
static constexpr int64_t g_patch_xcd_wbytes = 4 << 20;  // XCD grouping of the blocks: least weight bytes (0: never) ...
static constexpr int g_patch_xcd_rows = 16;              // ... and most row tiles
static bool patch_pick(int dt, int N, int dstH, int dstW, int srcC, int Ng, int R, int S, int stride, PatchShape& shape,
                       PatchArgs& geo) {
  if (R != 3 || S != 3 || stride != 1) return false;
  if (srcC % (dt == DT_F32 ? 16 : 32) != 0 || Ng % 64 != 0) return false;
  const int wide = Ng % 128 == 0 ? 128 : 64;
  // Candidates, largest first.  Two co-resident blocks per CU cover each other's prologue, barriers and epilogue, and
  // measured better than one block of twice the size at every layer of the benchmark networks, so the first
  // candidate that gives g_patch_fill (two per CU) blocks is taken, else the one with the most blocks.
  const PatchShape cand[3] = {{2, 1, wide, 1}, {2, 1, 64, 1}, {1, 1, 64, 1}};
  int best = -1;
  int64_t best_blocks = 0;
  PatchArgs best_geo{};
  for (int i = 0; i < 3; ++i) {
    if (!((g_patch_shapes >> i) & 1)) continue;
    if (i == 1 && wide == 64) continue;  // same as candidate 0
    const int cap = 64 * cand[i].mi / cand[i].subt;
    PatchArgs a{};
    if (!patch_geometry(N, dstH, dstW, cap, a)) continue;
    if (a.TP * 4 < cap * 3) continue;  // tile rows poorly used
    if (a.NPOS * 2 > a.TP * g_patch_halo2) continue;  // almost only halo: the staged patch costs more than it saves
    const int64_t blocks = (int64_t)((a.NT + cand[i].subt - 1) / cand[i].subt) * (Ng / cand[i].bn);
    if (blocks > best_blocks) { best = i; best_blocks = blocks; best_geo = a; }
    if (blocks >= g_patch_fill) break;
  }
  if (best < 0 || best_blocks < g_patch_min_blocks) return false;
  shape = cand[best];
  geo = best_geo;
  // still short of a block per CU: split the channel chunks over blockIdx.z (at least four chunks per range)
  const int nchunks = srcC / (dt == DT_F32 ? 16 : 32);
  int splits = 1;
  // fp32, smallest shape (one MFMA tile per wavefront, a barrier every 8 MFMAs): two co-resident blocks per CU
  // cover each other's barrier and LDS waits, which is worth the partial sums (measured 96 -> 84 us on 512->512 at 4x4)
  const int target = (shape.mi == 1 && dt == DT_F32) ? g_patch_target_small : 256;
  if (g_patch_split && best_blocks < target) {
    splits = (int)((target + best_blocks - 1) / best_blocks);
    if (splits > nchunks / 4) splits = nchunks / 4;
    if (splits > 4) splits = 4;
    if (splits < 1) splits = 1;
  }
  geo.row_pitch = patch_row_pitch(geo, shape.subt);
  geo.chunks_per_split = (nchunks + splits - 1) / splits;
  shape.splits = (nchunks + geo.chunks_per_split - 1) / geo.chunks_per_split;  // no empty ranges
  return true;
}

template <class T, int BN, int MI, int SUBT, bool FOLD>
static void launch_patch_v(hipStream_t st, const void* src, const void* wmat, const float* bias, const void* addend, void* out,
                           float* partial, float* stat_partial, int splits, const PatchArgs& a_in) {
  PatchArgs a = a_in;
  dim3 grid((a.NT + SUBT - 1) / SUBT, a.Ng / BN, splits), block(256);
  // The patch buffers are sized for this layer's tile (its staged rows times the row pitch), not for the largest one,
  // so that the 64-channel shapes fit three blocks per CU on most layers.  The epilogue reuses the buffers and the
  // weight stages: they must hold its fp32 tile and the 16 KB of the channel-sum combine.
  constexpr size_t sm_max = patch_smem_max<T>(BN, SUBT);
  constexpr int64_t PITCH_E = Frag<T>::BK + 16 / sizeof(T);
  const int64_t epi_bytes = std::max<int64_t>((int64_t)32 * MI * (BN + 4) * 4, 16384);
  int64_t pe = ((int64_t)SUBT * a.TI * a.SR * a.row_pitch + 15) / 16 * 16 / (int64_t)sizeof(T);
  const int64_t need = (epi_bytes - (int64_t)3 * BN * PITCH_E * (int64_t)sizeof(T) + 1) / 2;  // bytes per buffer
  if (pe * (int64_t)sizeof(T) < need) pe = (need + 15) / 16 * 16 / (int64_t)sizeof(T);
  if (pe > (int64_t)SUBT * PATCH_MAX_POS * PITCH_E) pe = (int64_t)SUBT * PATCH_MAX_POS * PITCH_E;
  a.patch_elems = (int)pe;
  // from the shape only: weights of at least g_patch_xcd_wbytes that at most g_patch_xcd_rows row tiles share
  a.xcd_group = g_patch_xcd_wbytes > 0 && (int64_t)9 * a.srcC * a.Ng * (int64_t)sizeof(T) >= g_patch_xcd_wbytes &&
                (int)grid.x <= g_patch_xcd_rows && (grid.y * grid.z) % 8 == 0;
  a.row_blocks = (int)grid.x;
  if (!a.xcd_group && grid.y * grid.z >= 2 && grid.x >= 64) {  // (from the shape only)
    a.xcd_group = 2;
    grid.x = (grid.x + 7) / 8 * 8;
  }
  const size_t sm = patch_smem_bytes<T>(BN, SUBT, pe);
  static bool attr_done = false;
  if (!attr_done) {
    (void)hipFuncSetAttribute((const void*)conv3x3_patch_kernel<T, BN, MI, SUBT, false, FOLD>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)sm_max);
    (void)hipFuncSetAttribute((const void*)conv3x3_patch_kernel<T, BN, MI, SUBT, true, FOLD>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)sm_max);
    attr_done = true;
  }
  // the variant that also adds up what it stores (BatchNorm statistics) is a separate instantiation, so that the
  // plain one carries none of its registers
  if (splits == 1 && stat_partial)
    OSEQ_LAUNCH((conv3x3_patch_kernel<T, BN, MI, SUBT, true, FOLD>), grid, block, sm, st, (const T*)src, (const T*)wmat, bias,
                       (const T*)addend, (T*)out, (float*)nullptr, stat_partial, a);
  else
    OSEQ_LAUNCH((conv3x3_patch_kernel<T, BN, MI, SUBT, false, FOLD>), grid, block, sm, st, (const T*)src, (const T*)wmat, bias,
                       (const T*)addend, (T*)out, splits > 1 ? partial : (float*)nullptr, (float*)nullptr, a);
}

template <class T>
static void launch_patch_t(hipStream_t st, const void* src, const void* wmat, const float* bias, const void* addend, void* out,
                           float* partial, float* stat_partial, const PatchShape& v, const PatchArgs& a) {
  const int sp = v.splits;
  if constexpr (sizeof(T) == 2) {
    if (a.fold) {  // (16-bit modes only)
      if (v.mi == 2) {
        if (v.bn == 128) launch_patch_v<T, 128, 2, 1, true>(st, src, wmat, bias, addend, out, partial, stat_partial, sp, a);
        else launch_patch_v<T, 64, 2, 1, true>(st, src, wmat, bias, addend, out, partial, stat_partial, sp, a);
      } else {
        launch_patch_v<T, 64, 1, 1, true>(st, src, wmat, bias, addend, out, partial, stat_partial, sp, a);
      }
    }
  }
  if (sizeof(T) != 2 || !a.fold) {
    if (v.mi == 2) {
      if (v.bn == 128) launch_patch_v<T, 128, 2, 1, false>(st, src, wmat, bias, addend, out, partial, stat_partial, sp, a);
      else launch_patch_v<T, 64, 2, 1, false>(st, src, wmat, bias, addend, out, partial, stat_partial, sp, a);
    } else {
      launch_patch_v<T, 64, 1, 1, false>(st, src, wmat, bias, addend, out, partial, stat_partial, sp, a);
    }
  }
  if (sp > 1)
    launch_splitk_epilogue<T>(st, partial, sp, (int64_t)a.N * a.dstH * a.dstW, a.Ng, bias, addend, a.amask, out, stat_partial, a.relu);
}

static void launch_patch(hipStream_t st, int dt, const void* src, const void* wmat, const float* bias, const void* addend, void* out,
                         float* partial, float* stat_partial, const PatchShape& v, const PatchArgs& a) {
  if (dt == DT_F32) launch_patch_t<float>(st, src, wmat, bias, addend, out, partial, stat_partial, v, a);
  else if (dt == DT_BF16) launch_patch_t<bf16_t>(st, src, wmat, bias, addend, out, partial, stat_partial, v, a);
  else launch_patch_t<f16_t>(st, src, wmat, bias, addend, out, partial, stat_partial, v, a);
}

static constexpr int g_igemm_spread = 1;                         // compile-time switch
constexpr size_t kSpreadLds = 84 * 1024;        // more than half of the 160 KB of LDS per CU

// Rows per block.  A 256-row tile was tried for layers with many pixels: it needs 348-380 registers, so one wavefront
// per SIMD, where two 128-row blocks share a CU; the strided 3x3 layers of the bottleneck network at batch 4096 (bf16)
// take 716 / 646 us with it and 551 / 520 without, the fp32 network on 512 x 512 images 166.4 against 163.2 ms a step.
constexpr int IGEMM_BM = 128;

template <class T, int MODE>
static void launch_igemm_t(hipStream_t st, const void* src, const void* wmat, const float* bias, const void* addend, void* out,
                           float* partial, float* stat_partial, int splits, const IGemmArgs& a0) {
  IGemmArgs a = a0;
  const int bk = Frag<T>::BK;
  a.kt_per_split = ceil_div(a.Kg / bk, splits);
  const bool wide = a.Ng % 128 == 0;
  dim3 grid(ceil_div(a.M, IGEMM_BM), a.Ng / (wide ? 128 : 64), a.cls ? 4 : splits), block(256);  // cls: never split
  // A grid of at most one block per CU asks for more than half of a CU's LDS, so that no CU takes two blocks
  // while another idles.
  const bool spread = g_igemm_spread && (int64_t)grid.x * grid.y * grid.z <= 256;
#define IGEMM_LAUNCH(BM_, BN_, SPLIT_)                                                                                   \
  {                                                                                                                      \
    constexpr size_t sm_ = igemm_smem_bytes<T, BM_, BN_>();                                                              \
    constexpr size_t big_ = sm_ > kSpreadLds ? sm_ : kSpreadLds;                                                         \
    static bool attr_ = false;                                                                                           \
    if (!attr_) {                                                                                                        \
      (void)hipFuncSetAttribute((const void*)conv_igemm_kernel<T, BM_, BN_, MODE, SPLIT_>,                               \
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)big_);                                  \
      attr_ = true;                                                                                                      \
    }                                                                                                                    \
    OSEQ_LAUNCH((conv_igemm_kernel<T, BM_, BN_, MODE, SPLIT_>), grid, block, spread ? big_ : sm_, st,             \
                       (const T*)src, (const T*)wmat, bias, (const T*)addend, (T*)out, partial, stat_partial, a);        \
  }
  if (splits > 1) {
    if (wide) IGEMM_LAUNCH(128, 128, true) else IGEMM_LAUNCH(128, 64, true)
    launch_splitk_epilogue<T>(st, partial, splits, a.M, a.Ng, bias, addend, a.amask, out, stat_partial, a.relu);
  } else {
    if (wide) IGEMM_LAUNCH(128, 128, false) else IGEMM_LAUNCH(128, 64, false)
  }
#undef IGEMM_LAUNCH
}

template <int MODE>
static void launch_igemm(hipStream_t st, int dt, const void* src, const void* wmat, const float* bias, const void* addend,
                         void* out, float* partial, float* stat_partial, int splits, const IGemmArgs& a) {
  if (dt == DT_F32) launch_igemm_t<float, MODE>(st, src, wmat, bias, addend, out, partial, stat_partial, splits, a);
  else if (dt == DT_BF16) launch_igemm_t<bf16_t, MODE>(st, src, wmat, bias, addend, out, partial, stat_partial, splits, a);
  else launch_igemm_t<f16_t, MODE>(st, src, wmat, bias, addend, out, partial, stat_partial, splits, a);
}

// depth splits of a GEMM with M rows, Ng columns and depth Kg: from the shape only
static int igemm_splits(int dt, int64_t M, int Ng, int Kg) {
  const int bk = dt == DT_F32 ? 16 : 32;
  const int64_t blocks = ((M + 127) / 128) * (Ng / (Ng % 128 == 0 ? 128 : 64));
  if (blocks >= 256) return 1;
  int64_t s = (512 + blocks - 1) / blocks;
  const int64_t most = (Kg / bk) / 8;  // at least eight depth tiles per range
  if (s > most) s = most;
  if (s > 32) s = 32;
  return (int)(s < 1 ? 1 : s);
}
int conv_mfma_fwd_splits(int dt, const ConvGeom& g) {
  PatchShape v; PatchArgs pa{};
  if (conv_pointwise_fwd_ok(dt, g)) return 1;
  if (patch_pick(dt, g.N, g.P, g.Q, g.C, g.K, g.R, g.S, g.stride, v, pa)) return v.splits;
  return igemm_splits(dt, (int64_t)g.N * g.P * g.Q, g.K, g.R * g.S * g.C);
}
// stride 2, even image, at most 3x3: the data gradient runs as four parity-class GEMMs in one launch
static constexpr int g_dgrad_classes = 1;  // compile-time switch
static bool dgrad_by_classes(const ConvGeom& g) {
  return g_dgrad_classes && g.stride == 2 && g.H % 2 == 0 && g.W % 2 == 0 && g.R <= 3 && g.S <= 3;
}
int conv_mfma_dgrad_splits(int dt, const ConvGeom& g) {
  PatchShape v; PatchArgs pa{};
  if (conv_pointwise_dgrad_ok(dt, g)) return 1;
  if (patch_pick(dt, g.N, g.H, g.W, g.K, g.C, g.R, g.S, g.stride, v, pa)) return v.splits;
  if (dgrad_by_classes(g)) return 1;
  return igemm_splits(dt, (int64_t)g.N * g.H * g.W, g.C, g.R * g.S * g.K);
}

bool conv_mfma_fwd_ok(int dt, const ConvGeom& g) {
  const int bk = dt == DT_F32 ? 16 : 32;
  return g.C % bk == 0 && g.K % 64 == 0;
}
bool conv_mfma_dgrad_ok(int dt, const ConvGeom& g) {
  const int bk = dt == DT_F32 ? 16 : 32;
  return g.K % bk == 0 && g.C % 64 == 0;
}

// Row blocks over which the forward path produces the per-channel sums for BatchNorm: the blocks of the convolution
// kernel, or of the kernel that adds the depth ranges when the depth is split.  From the layer shape only.
int conv_mfma_fwd_stat_blocks(int dt, const ConvGeom& g) {
  PatchShape pv; PatchArgs pa{};
  const int64_t M = (int64_t)g.N * g.P * g.Q;
  if (conv_pointwise_fwd_ok(dt, g)) return conv_pointwise_stat_blocks(g);
  if (patch_pick(dt, g.N, g.P, g.Q, g.C, g.K, g.R, g.S, g.stride, pv, pa))
    return pv.splits > 1 ? ceil_div(M, SPLIT_EPI_ROWS) : (pa.NT + pv.subt - 1) / pv.subt;
  if (igemm_splits(dt, M, g.K, g.R * g.S * g.C) > 1) return ceil_div(M, SPLIT_EPI_ROWS);
  return ceil_div(M, IGEMM_BM);
}

// stat_partial: null, or [conv_mfma_fwd_stat_blocks][2][C_out] floats receiving per-block sums and sums of squares
// of the stored outputs
// the 1x1 streaming kernels and, in the 16-bit modes, the 3x3 patch kernel
bool conv_fold_fwd_ok(int dt, const ConvGeom& g) {
  if (conv_pointwise_fwd_ok(dt, g)) return conv_pointwise_fold_ok(dt, g);
  PatchShape pv; PatchArgs pa{};
  return dt != DT_F32 && patch_pick(dt, g.N, g.P, g.Q, g.C, g.K, g.R, g.S, g.stride, pv, pa);
}

void launch_conv_fwd_mfma(hipStream_t st, int dt, const void* x, const void* w, const float* bias, void* out,
                          float* partial, float* stat_partial, int splits, const ConvGeom& g, int relu, const float* fold) {
  PatchShape pv; PatchArgs pa{};
  if (conv_pointwise_fwd_ok(dt, g)) {
    launch_conv_fwd_pointwise(st, dt, x, w, bias, out, stat_partial, g, relu, fold);
    return;
  }
  if (patch_pick(dt, g.N, g.P, g.Q, g.C, g.K, g.R, g.S, g.stride, pv, pa)) {
    pa.N = g.N; pa.srcH = g.H; pa.srcW = g.W; pa.srcC = g.C; pa.dstH = g.P; pa.dstW = g.Q; pa.Ng = g.K;
    pa.pad = g.pad; pa.flip = 0; pa.relu = relu;
    pa.fold = dt == DT_F32 ? nullptr : fold;
    launch_patch(st, dt, x, w, bias, nullptr, out, partial, stat_partial, pv, pa);
    return;
  }
  IGemmArgs a{g.H, g.W, g.C, g.P, g.Q, g.N * g.P * g.Q, g.K, g.R * g.S * g.C, g.R, g.S, g.stride, g.pad, relu, 0};
  launch_igemm<IG_FWD>(st, dt, x, w, bias, nullptr, out, partial, stat_partial, splits, a);
}

// wt: the (C_in, kh, kw, C_out) transpose of the weights, in the compute type
void launch_conv_dgrad_mfma(hipStream_t st, int dt, const void* dz, const void* wt, const void* addend,
                            const void* addend_mask, void* dx, float* partial, int splits, const ConvGeom& g) {
  PatchShape pv; PatchArgs pa{};
  const uint8_t* amask = addend ? (const uint8_t*)addend_mask : nullptr;
  if (conv_pointwise_dgrad_ok(dt, g)) {
    launch_conv_dgrad_pointwise(st, dt, dz, wt, addend, amask, dx, g);
    return;
  }
  if (patch_pick(dt, g.N, g.H, g.W, g.K, g.C, g.R, g.S, g.stride, pv, pa)) {
    pa.N = g.N; pa.srcH = g.P; pa.srcW = g.Q; pa.srcC = g.K; pa.dstH = g.H; pa.dstW = g.W; pa.Ng = g.C;
    pa.pad = g.R - 1 - g.pad; pa.flip = 1; pa.relu = 0; pa.amask = amask;
    launch_patch(st, dt, dz, wt, nullptr, addend, dx, partial, nullptr, pv, pa);
    return;
  }
  IGemmArgs a{g.P, g.Q, g.K, g.H, g.W, g.N * g.H * g.W, g.C, g.R * g.S * g.K, g.R, g.S, g.stride, g.pad, 0, 0};
  a.amask = amask;  // (only stride-1 layers ever get one: the identity shortcut of a block)
  if (dgrad_by_classes(g)) {
    a.cls = 1; a.fullH = g.H; a.fullW = g.W;
    a.dstH = g.H / 2; a.dstW = g.W / 2; a.M = g.N * a.dstH * a.dstW;
    for (int c = 0; c < 4; ++c) {
      const int ph = c >> 1, pw = c & 1;
      a.taps[c] = 0; a.ntaps[c] = 0;
      for (int r = 0; r < g.R; ++r)
        for (int s2 = 0; s2 < g.S; ++s2)
          if (((ph + g.pad - r) & 1) == 0 && ((pw + g.pad - s2) & 1) == 0)
            a.taps[c] |= (r * g.S + s2) << (8 * a.ntaps[c]++);
    }
    launch_igemm<IG_DGRAD>(st, dt, dz, wt, nullptr, addend, dx, nullptr, nullptr, 1, a);
    return;
  }
  launch_igemm<IG_DGRAD>(st, dt, dz, wt, nullptr, addend, dx, partial, nullptr, splits, a);
}

// (C_out, R*S, C_in) fp32 master weights -> (C_in, R*S, C_out) in the compute type, for all layers of a batch in one
// launch: a block transposes one 32x32 (C_out x C_in) tile of one filter tap through LDS, so that both the reads
// (along C_in) and the writes (along C_out) are contiguous.
template <class T>
__global__ void __launch_bounds__(256) weight_transpose_kernel(const float* __restrict__ wbase, T* __restrict__ wtbase,
                                                               TransposeBatch b) {
  __shared__ float tile[32][33];
  int j = 0;
  while (j + 1 < b.n && (int)blockIdx.x >= b.job[j + 1].first_block) ++j;
  const TransposeJob jb = b.job[j];
  const int tiles_k = (jb.K + 31) / 32, tiles_c = (jb.C + 31) / 32;
  const int local = blockIdx.x - jb.first_block;
  const int tc = local % tiles_c, t2 = local / tiles_c;
  const int tk = t2 % tiles_k, rs = t2 / tiles_k;
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
  const float* w = wbase + jb.w_off;
  T* wt = wtbase + jb.w_off;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int k = tk * 32 + ty + i * 8, c = tc * 32 + tx;
    if (k < jb.K && c < jb.C) tile[ty + i * 8][tx] = w[((int64_t)k * jb.RS + rs) * jb.C + c];
  }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int c = tc * 32 + ty + i * 8, k = tk * 32 + tx;
    if (c < jb.C && k < jb.K) wt[((int64_t)c * jb.RS + rs) * jb.K + k] = from_f32<T>(tile[tx][ty + i * 8]);
  }
}

// jobs: first_block is filled in here
void launch_weight_transposes(hipStream_t st, int dt, const float* wbase, void* wtbase, const TransposeJob* jobs, int njobs) {
  for (int j0 = 0; j0 < njobs; j0 += TransposeBatch::MAX_JOBS) {
    TransposeBatch b{};
    b.n = njobs - j0 < TransposeBatch::MAX_JOBS ? njobs - j0 : TransposeBatch::MAX_JOBS;
    int blocks = 0;
    for (int j = 0; j < b.n; ++j) {
      b.job[j] = jobs[j0 + j];
      b.job[j].first_block = blocks;
      blocks += b.job[j].RS * ((b.job[j].K + 31) / 32) * ((b.job[j].C + 31) / 32);
    }
    if (blocks == 0) continue;
    if (dt == DT_F32) OSEQ_LAUNCH(weight_transpose_kernel<float>, dim3(blocks), dim3(256), 0, st, wbase, (float*)wtbase, b);
    else if (dt == DT_BF16) OSEQ_LAUNCH(weight_transpose_kernel<bf16_t>, dim3(blocks), dim3(256), 0, st, wbase, (bf16_t*)wtbase, b);
    else OSEQ_LAUNCH(weight_transpose_kernel<f16_t>, dim3(blocks), dim3(256), 0, st, wbase, (f16_t*)wtbase, b);
  }
}

// ------------------------------------------------------------------------------------------------------------
// Weight gradient:  dw[k][tap][c] = sum over pixels m of dz[m][k] * x_tap[m][c]   (fp32 result)
// One block owns a (BM output channels) x (BN input channels) tile of ONE filter tap and a fixed chunk of the
// pixel range (blockIdx.z); chunks are summed afterwards in order, so the result does not depend on scheduling.
// Both operands arrive pixel-major (the reduction index is the slow one), but an MFMA lane wants consecutive
// reduction elements.  The tiles are stored in LDS exactly as loaded (16-byte chunks, [pixel][channel]); fp32 lanes
// read them with a stride, 16-bit lanes use the transposing LDS read of gfx950 (ds_read_b64_tr_b16).
// ------------------------------------------------------------------------------------------------------------
struct WGradArgs {
  int H, W, C, K, R, S, stride, pad, P, Q;
  int pixels, chunk;  // chunk: pixels per blockIdx.z, a multiple of the depth tile
  FastDiv divQ, divPQ;
  const float* fold;  // FOLD: x is the z of a BatchNorm + ReLU, this its [4][C] statistics tensor; the pieces of x become
                      // the activation (scale, shift, ReLU, one rounding) on their way to LDS
  int xcd_group;      // 1: the tiles of a pixel range share an XCD (see the kernel); ranges: the number of pixel ranges
  int ranges;
};

template <class T> struct WFrag;
template <> struct WFrag<float> {
  static constexpr int DEPTH = 16;  // pixels per depth tile
  float v[8];
  __device__ __forceinline__ void load(const float* tile, int pitch, int col, int g) {
#pragma unroll
    for (int t = 0; t < 8; ++t) v[t] = tile[(g * 8 + t) * pitch + col];
  }
  __device__ static __forceinline__ void mma(const WFrag& a, const WFrag& b, v16f& c) {
#pragma unroll
    for (int t = 0; t < 8; ++t) c = __builtin_amdgcn_mfma_f32_32x32x2f32(a.v[t], b.v[t], c, 0, 0, 0);
  }
};

typedef __attribute__((ext_vector_type(4))) short v4s;
typedef __attribute__((ext_vector_type(8))) short v8s;
// two transposing 64-bit LDS reads (see the weight-gradient kernel): 8 consecutive reduction elements of one channel
template <class T>
__device__ __forceinline__ v8s tr_read8(const T* p0, const T* p1) {
  const v4s a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) v4s*)(p0));
  const v4s b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) v4s*)(p1));
  v8s r = {a[0], a[1], a[2], a[3], b[0], b[1], b[2], b[3]};
  return r;
}

// WGM x WGN wavefronts (wave tile BM / WGM x BN / WGN); the 256 x 256 tile of the 1x1 layers with many pixels runs 2 x 4
// wavefronts, two per SIMD, one block per CU: every operand element then crosses from L2 to a CU half as often as with
// 128 x 128 tiles (a 1024 x 256 weight gradient over 262 144 pixels moves 1.07 GB instead of 2.1 GB that way).
template <class T, int BM, int BN, int WGM>
constexpr size_t wgrad_lds_bytes() {
  return (size_t)3 * (sizeof(T) == 4 ? 16 : 32) * (BM + BN + 2 * (sizeof(T) == 4 ? 4 : 16)) * sizeof(T);
}

// PW: a 1x1 layer with unit stride and no padding -- pixel m of x is row m, as it is of dz; the loads of a depth tile
// are then one uniform base per tensor plus per-thread offsets that never change (the general path divides every
// pixel index into image, row and column and multiplies it back into an address, a few dozen quarter-rate integer
// multiplies per depth tile that the 256 x 256 tile, with one block per CU, has nobody to hide behind).
// NTL (PW only): 1 / 2: the rows of dz / of x are read by this block's tile alone (one input- / output-channel tile) and
// are loaded non-temporally
template <class T, int BM, int BN, int WGM = 2, int WGN = 2, bool FOLD = false, bool PW = false, int NTL = 0>
__global__ void __launch_bounds__(64 * WGM * WGN) conv_wgrad_kernel(const T* __restrict__ x, const T* __restrict__ dz,
                                                                    float* __restrict__ out, WGradArgs a) {
  constexpr bool F32 = sizeof(T) == 4;
  constexpr int DEPTH = F32 ? 16 : 32;
  constexpr int NT = 64 * WGM * WGN;
  constexpr int WTM = BM / WGM, WTN = BN / WGN;
  constexpr int MI = WTM / 32, NI = WTN / 32;
  // one LDS stage, pixel-major exactly as loaded: [DEPTH][BM + pad] then [DEPTH][BN + pad] (pad: 4 floats / 16 halves)
  constexpr int PADE = F32 ? 4 : 16;
  constexpr int A_ELEMS = DEPTH * (BM + PADE);
  constexpr int B_ELEMS = DEPTH * (BN + PADE);
  constexpr int STAGE = A_ELEMS + B_ELEMS;
  extern __shared__ __attribute__((aligned(16))) unsigned char wgrad_smem[];
  T* lds = reinterpret_cast<T*>(wgrad_smem);

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WGN, wn = wave % WGN, g = lane >> 5, l32 = lane & 31;
  // Block coordinates: (output-channel tile, tap and input-channel tile, pixel range).  xcd_group (1x1 layers): the
  // tiles of one pixel range all read the same rows of x and dz; workgroups go to the 8 XCDs round-robin by their linear
  // index and every XCD has an L2 of its own, so the tiles of a range are renumbered onto one XCD, which then fetches
  // those rows once.  The grid's z extent is the number of ranges rounded up to a multiple of 8.
  int bx = blockIdx.x, by = blockIdx.y, bz = blockIdx.z;
  if (a.xcd_group) {
    const unsigned tiles = gridDim.x * gridDim.y;
    const unsigned lin = blockIdx.x + gridDim.x * (blockIdx.y + gridDim.y * blockIdx.z);
    const unsigned xcd = lin & 7u, slot = lin >> 3;
    const unsigned tile = slot % tiles;
    bz = (int)((slot / tiles) * 8u + xcd);
    bx = (int)(tile % gridDim.x); by = (int)(tile / gridDim.x);
    if (bz >= a.ranges) return;
  }
  const int k0 = bx * BM;
  const int ctiles = a.C / BN;
  const int tap = by / ctiles, c0 = (by - tap * ctiles) * BN;
  const int r = tap / a.S, s = tap - r * a.S;
  const int mbeg = bz * a.chunk;
  const int mend = mbeg + a.chunk < a.pixels ? mbeg + a.chunk : a.pixels;
  const int n = mend > mbeg ? (mend - mbeg + DEPTH - 1) / DEPTH : 0;
  const int K = a.K, C = a.C, H = a.H, W = a.W, cstride = a.stride, pad = a.pad;
  const FastDiv divQ = a.divQ, divPQ = a.divPQ;

  // staging: 16-byte chunks, rows = pixels (EV elements per chunk)
  constexpr int EV = 16 / (int)sizeof(T);
  constexpr int A_CH32 = DEPTH * (BM / EV) / NT, B_CH32 = DEPTH * (BN / EV) / NT;
  static_assert(A_CH32 >= 1 && B_CH32 >= 1, "tile too small for the block");
  Chunk ra[2][A_CH32], rb[2][B_CH32];
  unsigned va[2] = {0u, 0u}, vb[2] = {0u, 0u};  // validity bits of the pieces in flight, per generation

  // Loads are unconditional (pixels past the range or outside the image read pixel mbeg / the tensor start) and are
  // zeroed when written to LDS, so that later tiles' loads stay in flight during the MFMAs of the current one.
  auto tap_offset = [&](int n_, int p_, int q_, int64_t& off) -> bool {  // x offset of (image, row, col) under this tap
    const int ih = p_ * cstride + r - pad, iw = q_ * cstride + s - pad;
    const bool ok = ih >= 0 && ih < H && iw >= 0 && iw < W;
    off = ok ? (((int64_t)n_ * H + ih) * W + iw) * C : 0;
    return ok;
  };
  // PW: element offsets of a thread's pieces from the first row of a depth tile
  int offa[PW ? A_CH32 : 1], offb[PW ? B_CH32 : 1];
  if constexpr (PW) {
#pragma unroll
    for (int i = 0; i < A_CH32; ++i) {
      const int id = tid + i * NT, px = id / (BM / EV), kv = id % (BM / EV);
      offa[i] = px * K + k0 + kv * EV;
    }
#pragma unroll
    for (int i = 0; i < B_CH32; ++i) {
      const int id = tid + i * NT, px = id / (BN / EV), cv = id % (BN / EV);
      offb[i] = px * C + c0 + cv * EV;
    }
  }
  // CHK = 0: the tile is known to lie inside the range (every tile but a range's last one)
  auto gload = [&](auto G, auto CHKC, int t) {
    constexpr int p = decltype(G)::value;
    constexpr bool CHK = decltype(CHKC)::value != 0;
    const int mt = mbeg + t * DEPTH;
    unsigned ma = 0u, mb = 0u;
    if constexpr (PW) {
      const T* dzt = dz + (int64_t)mt * K;
      const T* xt = x + (int64_t)mt * C;
#pragma unroll
      for (int i = 0; i < A_CH32; ++i) {
        const int px = (tid + i * NT) / (BM / EV);
        const bool ok = !CHK || mt + px < mend;  // a row past the range reads the same piece of the range's first row
        const Chunk* pa = reinterpret_cast<const Chunk*>(ok ? dzt + offa[i] : dz + (int64_t)mbeg * K + (offa[i] - px * K));
        ra[p][i] = NTL == 1 ? __builtin_nontemporal_load(pa) : *pa;
        ma |= ok ? (1u << i) : 0u;
      }
#pragma unroll
      for (int i = 0; i < B_CH32; ++i) {
        const int px = (tid + i * NT) / (BN / EV);
        const bool ok = !CHK || mt + px < mend;
        const Chunk* pb = reinterpret_cast<const Chunk*>(ok ? xt + offb[i] : x + (int64_t)mbeg * C + (offb[i] - px * C));
        rb[p][i] = NTL == 2 ? __builtin_nontemporal_load(pb) : *pb;
        mb |= ok ? (1u << i) : 0u;
      }
      va[p] = ma; vb[p] = mb;
      return;
    }
#pragma unroll
    for (int i = 0; i < A_CH32; ++i) {
      const int id = tid + i * NT, px = id / (BM / EV), kv = id % (BM / EV);
      const int m = mt + px;
      const bool ok = m < mend;
      ra[p][i] = *reinterpret_cast<const Chunk*>(dz + (int64_t)(ok ? m : mbeg) * K + k0 + kv * EV);
      ma |= ok ? (1u << i) : 0u;
    }
#pragma unroll
    for (int i = 0; i < B_CH32; ++i) {
      const int id = tid + i * NT, px = id / (BN / EV), cv = id % (BN / EV);
      const int m = mt + px;
      const int mm = m < mend ? m : mbeg;
      const uint32_t n_ = divPQ.div((uint32_t)mm), rem = (uint32_t)mm - n_ * divPQ.d;
      const uint32_t p_ = divQ.div(rem), q_ = rem - p_ * divQ.d;
      int64_t off;
      const bool ok = tap_offset((int)n_, (int)p_, (int)q_, off) && m < mend;
      rb[p][i] = *reinterpret_cast<const Chunk*>(x + (ok ? off : 0) + c0 + cv * EV);
      mb |= ok ? (1u << i) : 0u;
    }
    va[p] = ma; vb[p] = mb;
  };
  // FOLD: a thread's pieces of x all cover the same EV channels, whose scale and shift it keeps in registers
  static_assert(NT % (BN / EV) == 0, "a thread's pieces of x must share their channels");
  float fsc[EV], fsh[EV];
  if (FOLD) {
    const int cv = tid % (BN / EV);
    load_f32<float, EV>(a.fold + 2 * C + c0 + cv * EV, fsc);
    load_f32<float, EV>(a.fold + 3 * C + c0 + cv * EV, fsh);
  }
  // FULL (PW only): every piece of the tile is known to be valid
  auto sstore = [&](auto G, auto FULLC, int stage) {
    constexpr int p = decltype(G)::value;
    constexpr bool FULL = PW && decltype(FULLC)::value != 0;
    T* sa = lds + stage * STAGE;
    T* sb = sa + A_ELEMS;
    if (FOLD) {
#pragma unroll
      for (int i = 0; i < B_CH32; ++i) rb[p][i] = bn_fold_chunk<T>(rb[p][i], fsc, fsh);
    }
#pragma unroll
    for (int i = 0; i < A_CH32; ++i) {
      const int id = tid + i * NT, px = id / (BM / EV), kv = id % (BM / EV);
      *reinterpret_cast<Chunk*>(&sa[px * (BM + PADE) + kv * EV]) = (FULL || ((va[p] >> i) & 1u)) ? ra[p][i] : zero_chunk();
    }
#pragma unroll
    for (int i = 0; i < B_CH32; ++i) {
      const int id = tid + i * NT, px = id / (BN / EV), cv = id % (BN / EV);
      *reinterpret_cast<Chunk*>(&sb[px * (BN + PADE) + cv * EV]) = (FULL || ((vb[p] >> i) & 1u)) ? rb[p][i] : zero_chunk();
    }
  };

  v16f acc[MI][NI];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NI; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  // operand registers: fp32 8 scalars per 32-row tile (pixels g*8 .. g*8+7 of the depth tile), 16-bit a 32-byte slice
  float fa32[F32 ? MI : 1][8], fb32[F32 ? NI : 1][8];
  Frag<T> fa[F32 ? 1 : MI], fb[F32 ? 1 : NI];
  const int acol = wm * WTM + l32, bcol = wn * WTN + l32;
  auto load_half = [&](int half, int stage) {
    const T* sa = lds + stage * STAGE;
    const T* sb = sa + A_ELEMS;
    if constexpr (F32) {
      const float* fsa = reinterpret_cast<const float*>(sa);
      const float* fsb = reinterpret_cast<const float*>(sb);
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        const int px = g * 8 + half * 4 + t;
#pragma unroll
        for (int i = 0; i < MI; ++i) fa32[i][half * 4 + t] = fsa[px * (BM + PADE) + acol + i * 32];
#pragma unroll
        for (int j = 0; j < NI; ++j) fb32[j][half * 4 + t] = fsb[px * (BN + PADE) + bcol + j * 32];
      }
    } else {
      // Transposing LDS read (ds_read_b64_tr_b16): within 16 lanes, lane r points at 4 consecutive channels of pixel
      // k0 + r/4 starting at channel 4*(r%4); lane l receives channel l of the 16 at pixels k0..k0+3.  Two reads give
      // the 8 pixels of one operand half for channel (tile base + l32).
      const int r16 = l32 & 15;
      const int kbase = g * 16 + half * 8 + (r16 >> 2);
      const int coff = (l32 & 16) + 4 * (r16 & 3);
#pragma unroll
      for (int i = 0; i < MI; ++i) {
        const T* pp = sa + kbase * (BM + PADE) + wm * WTM + i * 32 + coff;
        const v8s v = tr_read8(pp, pp + 4 * (BM + PADE));
        if (half == 0) fa[i].lo = __builtin_bit_cast(decltype(fa[i].lo), v); else fa[i].hi = __builtin_bit_cast(decltype(fa[i].hi), v);
      }
#pragma unroll
      for (int j = 0; j < NI; ++j) {
        const T* pp = sb + kbase * (BN + PADE) + wn * WTN + j * 32 + coff;
        const v8s v = tr_read8(pp, pp + 4 * (BN + PADE));
        if (half == 0) fb[j].lo = __builtin_bit_cast(decltype(fb[j].lo), v); else fb[j].hi = __builtin_bit_cast(decltype(fb[j].hi), v);
      }
    }
  };
  auto mma_half = [&](int half) {
    if constexpr (F32) {
#pragma unroll
      for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
          for (int j = 0; j < NI; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa32[i][half * 4 + t], fb32[j][half * 4 + t], acc[i][j], 0, 0, 0);
    } else {
#pragma unroll
      for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j) Frag<T>::mma_half(fa[i], fb[j], acc[i][j], half, 0);
    }
  };

  // pipeline as in the forward kernel: three LDS stages, two register generations, operand reload under the MFMAs
  if (n > 0) { gload(IC<0>{}, IC<1>{}, 0); sstore(IC<0>{}, IC<0>{}, 0); }
  if (n > 1) { gload(IC<1>{}, IC<1>{}, 1); sstore(IC<1>{}, IC<0>{}, 1); }
  if (n > 2) gload(IC<0>{}, IC<1>{}, 2);
  __syncthreads();
  if (n > 0) { load_half(0, 0); load_half(1, 0); }
  auto body = [&](auto G, auto TAILC, int j, int stage) {
    constexpr int p = decltype(G)::value;  // = j & 1: this generation holds tile j+2
    constexpr bool TAIL = decltype(TAILC)::value != 0;  // 0: steady state without range checks
    const int nstage = stage == 2 ? 0 : stage + 1;
    const bool has_next = TAIL ? j + 1 < n : true;
    // steady state (j + 4 < n): tiles j + 2 and j + 3 are not the range's last one, all of their rows are inside it
    if (!TAIL || j + 3 < n) gload(IC<1 - p>{}, IC<TAIL ? 1 : 0>{}, j + 3);
    mma_half(0);
    __builtin_amdgcn_sched_barrier(0);
    if (has_next) load_half(0, nstage);
    __builtin_amdgcn_sched_barrier(0);
    mma_half(1);
    __builtin_amdgcn_sched_barrier(0);
    if (has_next) load_half(1, nstage);
    if (!TAIL || j + 2 < n) sstore(G, IC<TAIL ? 0 : 1>{}, stage == 0 ? 2 : stage - 1);
    __syncthreads();
  };
  {
    int stage = 0, j = 0;
    for (; j + 4 < n; j += 2) {
      body(IC<0>{}, IC<0>{}, j, stage);
      stage = stage == 2 ? 0 : stage + 1;
      body(IC<1>{}, IC<0>{}, j + 1, stage);
      stage = stage == 2 ? 0 : stage + 1;
    }
    for (; j < n; j += 2) {
      body(IC<0>{}, IC<1>{}, j, stage);
      stage = stage == 2 ? 0 : stage + 1;
      if (j + 1 < n) {
        body(IC<1>{}, IC<1>{}, j + 1, stage);
        stage = stage == 2 ? 0 : stage + 1;
      }
    }
  }

  const int64_t outputs = (int64_t)K * a.R * a.S * C;
  float* dst = out + (int64_t)bz * outputs;
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NI; ++j) {
      const int c = c0 + wn * WTN + j * 32 + l32;
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int k = k0 + wm * WTM + i * 32 + 8 * (e >> 2) + 4 * g + (e & 3);
        dst[((int64_t)k * a.R * a.S + tap) * C + c] = acc[i][j][e];
      }
    }
}

bool conv_mfma_wgrad_ok(int dt, const ConvGeom& g) {
  (void)dt;
  return g.C % 64 == 0 && g.K % 64 == 0 && (int64_t)g.N * g.P * g.Q < (1 << 24) && g.P * g.Q < (1 << 24);
}

// number of pixel chunks, from the layer shape only
// 1x1 layers have only (K / 128) * (C / 128) tiles, often one or two, and hundreds of thousands of pixels: they take
// up to 256 pixel ranges and aim at two blocks per CU (measured on the 1x1 layers of ResNet-50 at batch 128, bf16:
// 64->64 at 56x56 64 -> 23 us, 64->256 91 -> 56 us, 256->128 126 -> 75 us, all fifteen layers 995 -> 743 us)
static constexpr int g_wgrad_blocks = 1024;  // compile-time constants
static constexpr int g_wgrad_max_splits = 64;
static constexpr int g_wgrad_blocks_1x1 = 512;
static constexpr int g_wgrad_max_splits_1x1 = 256;
// 1x1 layers in the 16-bit modes whose channel counts are multiples of 256 and that have at least 64 K pixels take the
// 256 x 256 tile: one block per CU (256 blocks), every pixel range at least 16 depth tiles long
static bool wgrad_large_ok(int dt, const ConvGeom& g) {
  return dt != DT_F32 && g.R * g.S == 1 && g.K % 256 == 0 && g.C % 256 == 0 && (int64_t)g.N * g.P * g.Q >= 65536;
}
static int wgrad_large_splits(const ConvGeom& g) {
  const int64_t tiles = (int64_t)(g.K / 256) * (g.C / 256);
  const int64_t pixels = (int64_t)g.N * g.P * g.Q;
  int64_t want = tiles >= 256 ? 1 : (256 + tiles / 2) / tiles;
  const int64_t most = pixels / (16 * 32);
  if (want > most) want = most;
  if (want > 256) want = 256;
  return (int)(want < 1 ? 1 : want);
}

int conv_mfma_wgrad_splits(int dt, const ConvGeom& g) {
  if (conv_wgrad3x3_ok(dt, g)) return conv_wgrad3x3_splits(dt, g);
  if (wgrad_large_ok(dt, g)) return wgrad_large_splits(g);
  const int depth = dt == DT_F32 ? 16 : 32;
  const int bm = g.K % 128 == 0 ? 128 : 64, bn = g.C % 128 == 0 ? 128 : 64;
  const int64_t tiles = (int64_t)(g.K / bm) * (g.C / bn) * g.R * g.S;
  const int64_t pixels = (int64_t)g.N * g.P * g.Q;
  const bool pointwise = g.R * g.S == 1;
  const int target = pointwise ? g_wgrad_blocks_1x1 : g_wgrad_blocks;
  const int cap = pointwise ? g_wgrad_max_splits_1x1 : g_wgrad_max_splits;
  int64_t want = (target + tiles / 2) / tiles;                     // aim at about that many blocks
  const int64_t most = (pixels + 4 * depth - 1) / (4 * depth);     // at least four depth tiles per chunk
  if (want > most) want = most;
  if (want > cap) want = cap;
  return (int)(want < 1 ? 1 : want);
}

template <class T, bool FOLD>
static void launch_wgrad_t(hipStream_t st, const void* x, const void* dz, float* dst, int splits, const ConvGeom& g,
                           const float* fold) {
  constexpr int depth = sizeof(T) == 4 ? 16 : 32;
  WGradArgs a;
  a.H = g.H; a.W = g.W; a.C = g.C; a.K = g.K; a.R = g.R; a.S = g.S; a.stride = g.stride; a.pad = g.pad; a.P = g.P; a.Q = g.Q;
  a.pixels = g.N * g.P * g.Q;
  int chunk = (a.pixels + splits - 1) / splits;
  a.chunk = (chunk + depth - 1) / depth * depth;
  a.divQ = make_fastdiv((uint32_t)g.Q);
  a.divPQ = make_fastdiv((uint32_t)(g.P * g.Q));
  a.fold = fold;
  a.ranges = splits;
  a.xcd_group = g.R * g.S == 1 && splits >= 8;
  const int gz = a.xcd_group ? (splits + 7) / 8 * 8 : splits;
  if constexpr (sizeof(T) == 2) {
    if (wgrad_large_ok(DT_BF16, g)) {
      constexpr size_t sm = wgrad_lds_bytes<T, 256, 256, 2>();
      static bool attr_done = false;
      if (!attr_done) {
        (void)hipFuncSetAttribute((const void*)conv_wgrad_kernel<T, 256, 256, 2, 4, FOLD, false>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)sm);
        (void)hipFuncSetAttribute((const void*)conv_wgrad_kernel<T, 256, 256, 2, 4, FOLD, true>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)sm);
        (void)hipFuncSetAttribute((const void*)conv_wgrad_kernel<T, 256, 256, 2, 4, FOLD, true, 1>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)sm);
        (void)hipFuncSetAttribute((const void*)conv_wgrad_kernel<T, 256, 256, 2, 4, FOLD, true, 2>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)sm);
        attr_done = true;
      }
      // rows of x = pixels of dz, and the row offsets fit 32 bits
      const bool pw = g.stride == 1 && g.pad == 0 && (int64_t)32 * std::max(g.K, g.C) < (1 << 30);
      if (pw && g.C == 256 && g.K > 256)
        OSEQ_LAUNCH((conv_wgrad_kernel<T, 256, 256, 2, 4, FOLD, true, 1>), dim3(g.K / 256, g.C / 256, gz), dim3(512), sm, st, (const T*)x,
                    (const T*)dz, dst, a);
      else if (pw && g.K == 256 && g.C > 256)
        OSEQ_LAUNCH((conv_wgrad_kernel<T, 256, 256, 2, 4, FOLD, true, 2>), dim3(g.K / 256, g.C / 256, gz), dim3(512), sm, st, (const T*)x,
                    (const T*)dz, dst, a);
      else if (pw)
        OSEQ_LAUNCH((conv_wgrad_kernel<T, 256, 256, 2, 4, FOLD, true>), dim3(g.K / 256, g.C / 256, gz), dim3(512), sm, st, (const T*)x,
                    (const T*)dz, dst, a);
      else
        OSEQ_LAUNCH((conv_wgrad_kernel<T, 256, 256, 2, 4, FOLD, false>), dim3(g.K / 256, g.C / 256, gz), dim3(512), sm, st, (const T*)x,
                    (const T*)dz, dst, a);
      return;
    }
  }
  const bool m128 = g.K % 128 == 0, n128 = g.C % 128 == 0;
  const int bm = m128 ? 128 : 64, bn = n128 ? 128 : 64;
  dim3 grid(g.K / bm, g.R * g.S * (g.C / bn), gz), block(256);
  // 1x1, unit stride, no padding: rows of x = pixels of dz, and the row offsets fit 32 bits
  const bool pw = g.R * g.S == 1 && g.stride == 1 && g.pad == 0 && (int64_t)32 * std::max(g.K, g.C) < (1 << 30);
#define WGRAD_LAUNCH(BM_, BN_)                                                                                              \
  {                                                                                                                         \
    if (pw) OSEQ_LAUNCH((conv_wgrad_kernel<T, BM_, BN_, 2, 2, FOLD, true>), grid, block, (wgrad_lds_bytes<T, BM_, BN_, 2>()), st, \
                        (const T*)x, (const T*)dz, dst, a);                                                                 \
    else OSEQ_LAUNCH((conv_wgrad_kernel<T, BM_, BN_, 2, 2, FOLD, false>), grid, block, (wgrad_lds_bytes<T, BM_, BN_, 2>()), st,  \
                     (const T*)x, (const T*)dz, dst, a);                                                                    \
  }
  if (m128 && n128) WGRAD_LAUNCH(128, 128)
  else if (m128) WGRAD_LAUNCH(128, 64)
  else if (n128) WGRAD_LAUNCH(64, 128)
  else WGRAD_LAUNCH(64, 64)
#undef WGRAD_LAUNCH
}

// out[i] = sum over pixel ranges s of partial[s][i], in a fixed order: G groups of threads each add the ranges
// s = g, g + G, ... for the same four outputs, then the G sums are added in group order.  G grows with the number
// of ranges so that small weight tensors with many ranges still fill the chip.
template <int G>
__global__ void __launch_bounds__(256) wgrad_reduce_kernel(const float* __restrict__ partial, float* __restrict__ out, int64_t n,
                                                           int splits) {
  constexpr int QB = 256 / G;  // output quads per block
  __shared__ v4f red[G > 1 ? 256 : 1];
  const int ql = threadIdx.x % QB, sg = threadIdx.x / QB;
  const int64_t i = ((int64_t)blockIdx.x * QB + ql) * 4;
  const bool on = i < n;
  v4f acc = {0.f, 0.f, 0.f, 0.f};
  if (on) {
#pragma unroll 4
    for (int s = sg; s < splits; s += G) acc += *reinterpret_cast<const v4f*>(partial + (int64_t)s * n + i);
  }
  if constexpr (G > 1) {
    red[threadIdx.x] = acc;
    __syncthreads();
    if (sg == 0 && on) {
      v4f t = red[ql];
#pragma unroll
      for (int g = 1; g < G; ++g) t += red[g * QB + ql];
      *reinterpret_cast<v4f*>(out + i) = t;
    }
  } else {
    if (on) *reinterpret_cast<v4f*>(out + i) = acc;
  }
}

static void launch_wgrad_reduce(hipStream_t st, const float* partial, float* out, int64_t n, int splits) {
  const int64_t quads = n / 4;  // n is a multiple of 4 (C % 64 == 0)
  if (splits >= 64 || (splits >= 16 && quads < 65536))
    OSEQ_LAUNCH(wgrad_reduce_kernel<16>, dim3(ceil_div(quads, 16)), dim3(256), 0, st, partial, out, n, splits);
  else if (splits >= 8)
    OSEQ_LAUNCH(wgrad_reduce_kernel<4>, dim3(ceil_div(quads, 64)), dim3(256), 0, st, partial, out, n, splits);
  else
    OSEQ_LAUNCH(wgrad_reduce_kernel<1>, dim3(ceil_div(quads, 256)), dim3(256), 0, st, partial, out, n, splits);
}

// the matrix-core kernels in the 16-bit modes
bool conv_fold_wgrad_ok(int dt, const ConvGeom& g) { return dt != DT_F32 && conv_mfma_wgrad_ok(dt, g); }

void launch_conv_wgrad_mfma(hipStream_t st, int dt, const void* x, const void* dz, float* dw, float* partial, int splits,
                            const ConvGeom& g, const float* fold) {
  float* dst = splits > 1 ? partial : dw;
  if (conv_wgrad3x3_ok(dt, g)) launch_conv_wgrad3x3(st, dt, x, dz, dst, g, fold);  // splits == conv_wgrad3x3_splits(dt, g)
  else if (dt == DT_F32) launch_wgrad_t<float, false>(st, x, dz, dst, splits, g, nullptr);
  else if (dt == DT_BF16) {
    if (fold) launch_wgrad_t<bf16_t, true>(st, x, dz, dst, splits, g, fold);
    else launch_wgrad_t<bf16_t, false>(st, x, dz, dst, splits, g, nullptr);
  } else {
    if (fold) launch_wgrad_t<f16_t, true>(st, x, dz, dst, splits, g, fold);
    else launch_wgrad_t<f16_t, false>(st, x, dz, dst, splits, g, nullptr);
  }
  if (splits > 1) {
    launch_wgrad_reduce(st, partial, dw, (int64_t)g.K * g.R * g.S * g.C, splits);
  }
}

}  // namespace oseq
