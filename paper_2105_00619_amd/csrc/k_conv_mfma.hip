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
#include "dev_common.h"
#include "kernels.h"

namespace oseq {

typedef __attribute__((ext_vector_type(16))) float v16f;
typedef __attribute__((ext_vector_type(8))) __bf16 v8bf;
typedef __attribute__((ext_vector_type(8))) _Float16 v8h;
typedef __attribute__((ext_vector_type(4))) float v4f;

struct alignas(16) Chunk { uint32_t w[4]; };

enum { IG_FWD = 0, IG_DGRAD = 1 };

struct IGemmArgs {
  int srcH, srcW, srcC;   // gathered tensor
  int dstH, dstW;         // pixel grid of the result
  int M, Ng, Kg;          // GEMM sizes: rows (pixels), columns (channels), depth (R*S*srcC)
  int R, S, stride, pad, relu;
};

template <class T> struct Frag;  // 32 bytes of one operand row, and the MFMAs that consume it
template <> struct Frag<float> {
  static constexpr int BK = 16;
  v4f lo, hi;
  __device__ __forceinline__ void load(const float* p) { lo = *(const v4f*)p; hi = *(const v4f*)(p + 4); }
  static constexpr int lane_off(int g) { return g * 8; }
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
  static constexpr int lane_off(int g) { return g * 16; }
  __device__ static __forceinline__ void mma(const Frag& a, const Frag& b, v16f& c) {
    c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.lo, b.lo, c, 0, 0, 0);
    c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.hi, b.hi, c, 0, 0, 0);
  }
};
template <> struct Frag<f16_t> {
  static constexpr int BK = 32;
  v8h lo, hi;
  __device__ __forceinline__ void load(const f16_t* p) { lo = *(const v8h*)p; hi = *(const v8h*)(p + 8); }
  static constexpr int lane_off(int g) { return g * 16; }
  __device__ static __forceinline__ void mma(const Frag& a, const Frag& b, v16f& c) {
    c = __builtin_amdgcn_mfma_f32_32x32x16_f16(a.lo, b.lo, c, 0, 0, 0);
    c = __builtin_amdgcn_mfma_f32_32x32x16_f16(a.hi, b.hi, c, 0, 0, 0);
  }
};
// Within a depth tile the two lane groups (lanes 0-31, 32-63) own disjoint halves of the depth range and every MFMA
// pairs the same depth indices of A and B, so any assignment of depth indices to (lane group, step) gives the same sum.

template <class T, int BN, int MODE>
__global__ void __launch_bounds__(256) conv_igemm_kernel(const T* __restrict__ src, const T* __restrict__ wmat,
                                                         const float* __restrict__ bias, const T* __restrict__ addend,
                                                         T* __restrict__ out, IGemmArgs a) {
  constexpr int BM = 128;
  constexpr int BK = Frag<T>::BK;
  constexpr int EV = 16 / (int)sizeof(T);   // elements per 16-byte chunk
  constexpr int PITCH = BK + EV;            // LDS row pitch in elements (80 bytes)
  constexpr int NI = BN / 64;               // 32-column MFMA tiles per wavefront
  constexpr int A_CH = BM * 4 / 256;        // 16-byte chunks per thread and depth tile (4 chunks per row)
  constexpr int B_CH = BN * 4 / 256;
  __shared__ T As[2][BM * PITCH];
  __shared__ T Bs[2][BN * PITCH];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1, g = lane >> 5, l32 = lane & 31;
  const int m0 = blockIdx.x * BM, n0 = blockIdx.y * BN;
  const int vec = tid & 3, row0 = tid >> 2;  // this thread's chunk column and first row

  // pixel coordinates of this thread's A rows
  int pn[A_CH], pa[A_CH], pb[A_CH];
  bool prow[A_CH];
#pragma unroll
  for (int i = 0; i < A_CH; ++i) {
    const int m = m0 + row0 + i * 64;
    prow[i] = m < a.M;
    const int mm = prow[i] ? m : 0;
    pb[i] = mm % a.dstW;
    const int t = mm / a.dstW;
    pa[i] = t % a.dstH;
    pn[i] = t / a.dstH;
  }
  const T* brow[B_CH];
#pragma unroll
  for (int i = 0; i < B_CH; ++i) brow[i] = wmat + (int64_t)(n0 + row0 + i * 64) * a.Kg + vec * EV;

  Chunk ra[A_CH], rb[B_CH];
  auto gload = [&](int kt) {
    const int kk0 = kt * BK;
    const int tap = kk0 / a.srcC, c0 = kk0 - tap * a.srcC;
    const int r = tap / a.S, s = tap - r * a.S;
#pragma unroll
    for (int i = 0; i < A_CH; ++i) {
      int y, x;
      bool ok = prow[i];
      if (MODE == IG_FWD) {
        y = pa[i] * a.stride + r - a.pad;
        x = pb[i] * a.stride + s - a.pad;
      } else {
        const int ty = pa[i] + a.pad - r, tx = pb[i] + a.pad - s;
        ok = ok && ty >= 0 && tx >= 0;
        if (a.stride == 2) { ok = ok && !((ty | tx) & 1); y = ty >> 1; x = tx >> 1; } else { y = ty; x = tx; }
      }
      ok = ok && y >= 0 && y < a.srcH && x >= 0 && x < a.srcW;
      if (ok) ra[i] = *reinterpret_cast<const Chunk*>(src + (((int64_t)pn[i] * a.srcH + y) * a.srcW + x) * a.srcC + c0 + vec * EV);
      else ra[i] = Chunk{{0u, 0u, 0u, 0u}};
    }
#pragma unroll
    for (int i = 0; i < B_CH; ++i) rb[i] = *reinterpret_cast<const Chunk*>(brow[i] + kk0);
  };
  auto sstore = [&](int buf) {
#pragma unroll
    for (int i = 0; i < A_CH; ++i) *reinterpret_cast<Chunk*>(&As[buf][(row0 + i * 64) * PITCH + vec * EV]) = ra[i];
#pragma unroll
    for (int i = 0; i < B_CH; ++i) *reinterpret_cast<Chunk*>(&Bs[buf][(row0 + i * 64) * PITCH + vec * EV]) = rb[i];
  };

  v16f acc[2][NI];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < NI; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  const int nkt = a.Kg / BK;
  gload(0);
  sstore(0);
  __syncthreads();
  for (int kt = 0; kt < nkt; ++kt) {
    const int buf = kt & 1;
    if (kt + 1 < nkt) gload(kt + 1);
    Frag<T> fa[2], fb[NI];
#pragma unroll
    for (int i = 0; i < 2; ++i) fa[i].load(&As[buf][(wm * 64 + i * 32 + l32) * PITCH + Frag<T>::lane_off(g)]);
#pragma unroll
    for (int j = 0; j < NI; ++j) fb[j].load(&Bs[buf][(wn * (BN / 2) + j * 32 + l32) * PITCH + Frag<T>::lane_off(g)]);
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < NI; ++j) Frag<T>::mma(fa[i], fb[j], acc[i][j]);
    if (kt + 1 < nkt) sstore(buf ^ 1);
    __syncthreads();
  }

  // epilogue: accumulator element e of lane (g, l32) is row 8*(e/4) + 4*g + e%4, column l32 of its 32x32 tile
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < NI; ++j) {
      const int col = n0 + wn * (BN / 2) + j * 32 + l32;
      const float bv = bias ? bias[col] : 0.f;
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int row = m0 + wm * 64 + i * 32 + 8 * (e >> 2) + 4 * g + (e & 3);
        if (row < a.M) {
          const int64_t o = (int64_t)row * a.Ng + col;
          float v = acc[i][j][e] + bv;
          if (addend) v += to_f32(addend[o]);
          if (a.relu) v = fmaxf(v, 0.f);
          out[o] = from_f32<T>(v);
        }
      }
    }
}

template <class T, int MODE>
static void launch_igemm_t(hipStream_t st, const void* src, const void* wmat, const float* bias, const void* addend, void* out,
                           const IGemmArgs& a) {
  if (a.Ng % 128 == 0) {
    dim3 grid(ceil_div(a.M, 128), a.Ng / 128);
    hipLaunchKernelGGL((conv_igemm_kernel<T, 128, MODE>), grid, dim3(256), 0, st, (const T*)src, (const T*)wmat, bias,
                       (const T*)addend, (T*)out, a);
  } else {
    dim3 grid(ceil_div(a.M, 128), a.Ng / 64);
    hipLaunchKernelGGL((conv_igemm_kernel<T, 64, MODE>), grid, dim3(256), 0, st, (const T*)src, (const T*)wmat, bias,
                       (const T*)addend, (T*)out, a);
  }
}

template <int MODE>
static void launch_igemm(hipStream_t st, int dt, const void* src, const void* wmat, const float* bias, const void* addend,
                         void* out, const IGemmArgs& a) {
  if (dt == DT_F32) launch_igemm_t<float, MODE>(st, src, wmat, bias, addend, out, a);
  else if (dt == DT_BF16) launch_igemm_t<bf16_t, MODE>(st, src, wmat, bias, addend, out, a);
  else launch_igemm_t<f16_t, MODE>(st, src, wmat, bias, addend, out, a);
}

bool conv_mfma_fwd_ok(int dt, const ConvGeom& g) {
  const int bk = dt == DT_F32 ? 16 : 32;
  return g.C % bk == 0 && g.K % 64 == 0;
}
bool conv_mfma_dgrad_ok(int dt, const ConvGeom& g) {
  const int bk = dt == DT_F32 ? 16 : 32;
  return g.K % bk == 0 && g.C % 64 == 0;
}

void launch_conv_fwd_mfma(hipStream_t st, int dt, const void* x, const void* w, const float* bias, void* out,
                          const ConvGeom& g, int relu) {
  IGemmArgs a{g.H, g.W, g.C, g.P, g.Q, g.N * g.P * g.Q, g.K, g.R * g.S * g.C, g.R, g.S, g.stride, g.pad, relu};
  launch_igemm<IG_FWD>(st, dt, x, w, bias, nullptr, out, a);
}

// wt: the (C_in, kh, kw, C_out) transpose of the weights, in the compute type
void launch_conv_dgrad_mfma(hipStream_t st, int dt, const void* dz, const void* wt, const void* addend, void* dx,
                            const ConvGeom& g) {
  IGemmArgs a{g.P, g.Q, g.K, g.H, g.W, g.N * g.H * g.W, g.C, g.R * g.S * g.K, g.R, g.S, g.stride, g.pad, 0};
  launch_igemm<IG_DGRAD>(st, dt, dz, wt, nullptr, addend, dx, a);
}

// (C_out, R*S, C_in) fp32 master weights -> (C_in, R*S, C_out) in the compute type
template <class T>
__global__ void weight_transpose_kernel(const float* __restrict__ w, T* __restrict__ wt, int K, int RS, int C) {
  const int64_t total = (int64_t)K * RS * C;
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= total) return;
  const int k = (int)(i % K);
  const int64_t t = i / K;
  const int rs = (int)(t % RS);
  const int c = (int)(t / RS);
  wt[i] = from_f32<T>(w[((int64_t)k * RS + rs) * C + c]);
}

void launch_weight_transpose(hipStream_t st, int dt, const float* w, void* wt, int K, int RS, int C) {
  const int64_t total = (int64_t)K * RS * C;
  dim3 grid(ceil_div(total, 256)), block(256);
  if (dt == DT_F32) hipLaunchKernelGGL(weight_transpose_kernel<float>, grid, block, 0, st, w, (float*)wt, K, RS, C);
  else if (dt == DT_BF16) hipLaunchKernelGGL(weight_transpose_kernel<bf16_t>, grid, block, 0, st, w, (bf16_t*)wt, K, RS, C);
  else hipLaunchKernelGGL(weight_transpose_kernel<f16_t>, grid, block, 0, st, w, (f16_t*)wt, K, RS, C);
}

}  // namespace oseq
