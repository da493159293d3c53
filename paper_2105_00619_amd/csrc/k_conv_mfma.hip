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
  int kt_per_split;       // depth tiles per blockIdx.z when the depth is split
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

// SPLIT: blockIdx.z owns a fixed range of depth tiles and writes raw fp32 sums to partial[z][M][Ng]; a second
// kernel adds the ranges in order and applies the epilogue (layers with few output pixels, to fill the chip).
template <class T, int BN, int MODE, bool SPLIT>
__global__ void __launch_bounds__(256) conv_igemm_kernel(const T* __restrict__ src, const T* __restrict__ wmat,
                                                         const float* __restrict__ bias, const T* __restrict__ addend,
                                                         T* __restrict__ out, float* __restrict__ partial, IGemmArgs a) {
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

  const int kt0 = SPLIT ? blockIdx.z * a.kt_per_split : 0;
  const int nkt = SPLIT ? (kt0 + a.kt_per_split < a.Kg / BK ? kt0 + a.kt_per_split : a.Kg / BK) : a.Kg / BK;
  if (kt0 < nkt) {
    gload(kt0);
    sstore(kt0 & 1);
  }
  __syncthreads();
  for (int kt = kt0; kt < nkt; ++kt) {
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
          if (SPLIT) {
            partial[(int64_t)blockIdx.z * a.M * a.Ng + o] = acc[i][j][e];
          } else {
            float v = acc[i][j][e] + bv;
            if (addend) v += to_f32(addend[o]);
            if (a.relu) v = fmaxf(v, 0.f);
            out[o] = from_f32<T>(v);
          }
        }
      }
    }
}

template <class T>
__global__ void __launch_bounds__(256) splitk_epilogue_kernel(const float* __restrict__ partial, int splits, int64_t n, int Ng,
                                                              const float* __restrict__ bias, const T* __restrict__ addend,
                                                              T* __restrict__ out, int relu) {
  const int64_t i = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) * 4;
  if (i >= n) return;
  v4f acc = *reinterpret_cast<const v4f*>(partial + i);
  for (int z = 1; z < splits; ++z) acc += *reinterpret_cast<const v4f*>(partial + (int64_t)z * n + i);
  const int col = (int)(i % Ng);
  float r[4];
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    float v = acc[e];
    if (bias) v += bias[col + e];
    if (addend) v += to_f32(addend[i + e]);
    r[e] = relu ? fmaxf(v, 0.f) : v;
  }
  store_f32<T, 4>(out + i, r);
}

template <class T, int MODE>
static void launch_igemm_t(hipStream_t st, const void* src, const void* wmat, const float* bias, const void* addend, void* out,
                           float* partial, int splits, const IGemmArgs& a0) {
  IGemmArgs a = a0;
  const int bk = Frag<T>::BK;
  a.kt_per_split = ceil_div(a.Kg / bk, splits);
  const bool wide = a.Ng % 128 == 0;
  dim3 grid(ceil_div(a.M, 128), a.Ng / (wide ? 128 : 64), splits), block(256);
  if (splits > 1) {
    if (wide) hipLaunchKernelGGL((conv_igemm_kernel<T, 128, MODE, true>), grid, block, 0, st, (const T*)src, (const T*)wmat, bias, (const T*)addend, (T*)out, partial, a);
    else hipLaunchKernelGGL((conv_igemm_kernel<T, 64, MODE, true>), grid, block, 0, st, (const T*)src, (const T*)wmat, bias, (const T*)addend, (T*)out, partial, a);
    const int64_t n = (int64_t)a.M * a.Ng;  // a multiple of 4: Ng % 64 == 0
    hipLaunchKernelGGL(splitk_epilogue_kernel<T>, dim3(ceil_div(n / 4, 256)), dim3(256), 0, st, partial, splits, n, a.Ng, bias,
                       (const T*)addend, (T*)out, a.relu);
  } else {
    if (wide) hipLaunchKernelGGL((conv_igemm_kernel<T, 128, MODE, false>), grid, block, 0, st, (const T*)src, (const T*)wmat, bias, (const T*)addend, (T*)out, partial, a);
    else hipLaunchKernelGGL((conv_igemm_kernel<T, 64, MODE, false>), grid, block, 0, st, (const T*)src, (const T*)wmat, bias, (const T*)addend, (T*)out, partial, a);
  }
}

template <int MODE>
static void launch_igemm(hipStream_t st, int dt, const void* src, const void* wmat, const float* bias, const void* addend,
                         void* out, float* partial, int splits, const IGemmArgs& a) {
  if (dt == DT_F32) launch_igemm_t<float, MODE>(st, src, wmat, bias, addend, out, partial, splits, a);
  else if (dt == DT_BF16) launch_igemm_t<bf16_t, MODE>(st, src, wmat, bias, addend, out, partial, splits, a);
  else launch_igemm_t<f16_t, MODE>(st, src, wmat, bias, addend, out, partial, splits, a);
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
int conv_mfma_fwd_splits(int dt, const ConvGeom& g) { return igemm_splits(dt, (int64_t)g.N * g.P * g.Q, g.K, g.R * g.S * g.C); }
int conv_mfma_dgrad_splits(int dt, const ConvGeom& g) { return igemm_splits(dt, (int64_t)g.N * g.H * g.W, g.C, g.R * g.S * g.K); }

bool conv_mfma_fwd_ok(int dt, const ConvGeom& g) {
  const int bk = dt == DT_F32 ? 16 : 32;
  return g.C % bk == 0 && g.K % 64 == 0;
}
bool conv_mfma_dgrad_ok(int dt, const ConvGeom& g) {
  const int bk = dt == DT_F32 ? 16 : 32;
  return g.K % bk == 0 && g.C % 64 == 0;
}

void launch_conv_fwd_mfma(hipStream_t st, int dt, const void* x, const void* w, const float* bias, void* out,
                          float* partial, int splits, const ConvGeom& g, int relu) {
  IGemmArgs a{g.H, g.W, g.C, g.P, g.Q, g.N * g.P * g.Q, g.K, g.R * g.S * g.C, g.R, g.S, g.stride, g.pad, relu, 0};
  launch_igemm<IG_FWD>(st, dt, x, w, bias, nullptr, out, partial, splits, a);
}

// wt: the (C_in, kh, kw, C_out) transpose of the weights, in the compute type
void launch_conv_dgrad_mfma(hipStream_t st, int dt, const void* dz, const void* wt, const void* addend, void* dx,
                            float* partial, int splits, const ConvGeom& g) {
  IGemmArgs a{g.P, g.Q, g.K, g.H, g.W, g.N * g.H * g.W, g.C, g.R * g.S * g.K, g.R, g.S, g.stride, g.pad, 0, 0};
  launch_igemm<IG_DGRAD>(st, dt, dz, wt, nullptr, addend, dx, partial, splits, a);
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

// ------------------------------------------------------------------------------------------------------------
// Weight gradient:  dw[k][tap][c] = sum over pixels m of dz[m][k] * x_tap[m][c]   (fp32 result)
// One block owns a (BM output channels) x (BN input channels) tile of ONE filter tap and a fixed chunk of the
// pixel range (blockIdx.z); chunks are summed afterwards in order, so the result does not depend on scheduling.
// Both operands arrive pixel-major (the reduction index is the slow one), but an MFMA lane wants consecutive
// reduction elements.  fp32: the tile is stored as loaded and lanes read it with a stride.  16-bit: each thread
// loads two channels of several consecutive pixels, interleaves them in registers (byte permutes) and stores
// channel-major rows, so the MFMA operands are read exactly as in the forward kernel.
// ------------------------------------------------------------------------------------------------------------
struct FastDiv {  // floor(m / d) for m * d < 2^48
  uint64_t magic; uint32_t d;
  __device__ __forceinline__ uint32_t div(uint32_t m) const { return (uint32_t)(((uint64_t)m * magic) >> 48); }
};
static FastDiv make_fastdiv(uint32_t d) { FastDiv f; f.d = d; f.magic = (((uint64_t)1 << 48) + d - 1) / d; return f; }

struct WGradArgs {
  int H, W, C, K, R, S, stride, pad, P, Q;
  int pixels, chunk;  // chunk: pixels per blockIdx.z, a multiple of the depth tile
  FastDiv divQ, divPQ;
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

__device__ __forceinline__ uint32_t pack_lo(uint32_t a, uint32_t b) { return __builtin_amdgcn_perm(b, a, 0x05040100u); }
__device__ __forceinline__ uint32_t pack_hi(uint32_t a, uint32_t b) { return __builtin_amdgcn_perm(b, a, 0x07060302u); }

template <class T, int BM, int BN>
__global__ void __launch_bounds__(256) conv_wgrad_kernel(const T* __restrict__ x, const T* __restrict__ dz,
                                                         float* __restrict__ out, WGradArgs a) {
  constexpr bool F32 = sizeof(T) == 4;
  constexpr int DEPTH = F32 ? 16 : 32;
  constexpr int MI = BM / 64, NI = BN / 64;
  // fp32: tiles [DEPTH][BM+4] floats; 16-bit: tiles [BM][DEPTH+8] halves (80-byte rows)
  constexpr int A_ELEMS = F32 ? DEPTH * (BM + 4) : BM * (DEPTH + 8);
  constexpr int B_ELEMS = F32 ? DEPTH * (BN + 4) : BN * (DEPTH + 8);
  __shared__ __attribute__((aligned(16))) T As[2][A_ELEMS];
  __shared__ __attribute__((aligned(16))) T Bs[2][B_ELEMS];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1, g = lane >> 5, l32 = lane & 31;
  const int k0 = blockIdx.x * BM;
  const int ctiles = a.C / BN;
  const int tap = blockIdx.y / ctiles, c0 = (blockIdx.y - tap * ctiles) * BN;
  const int r = tap / a.S, s = tap - r * a.S;
  const int mbeg = blockIdx.z * a.chunk;
  const int mend = mbeg + a.chunk < a.pixels ? mbeg + a.chunk : a.pixels;
  const int ntiles = mend > mbeg ? (mend - mbeg + DEPTH - 1) / DEPTH : 0;

  // ---- fp32 staging: 16-byte chunks, rows = pixels --------------------------------------------------------
  constexpr int A_CH32 = DEPTH * (BM / 4) / 256 > 0 ? DEPTH * (BM / 4) / 256 : 1;
  constexpr int B_CH32 = DEPTH * (BN / 4) / 256 > 0 ? DEPTH * (BN / 4) / 256 : 1;
  // ---- 16-bit staging: each thread owns a channel pair and PXA / PXB consecutive pixels ---------------------
  constexpr int PXA = BM / 16, PXB = BN / 16;
  Chunk ra[F32 ? A_CH32 : 1], rb[F32 ? B_CH32 : 1];
  uint32_t ha[F32 ? 1 : PXA], hb[F32 ? 1 : PXB];

  auto src_pixel = [&](int m, int64_t& off) -> bool {  // x offset (elements) of pixel m under this block's tap
    if (m >= mend) return false;
    const uint32_t n = a.divPQ.div((uint32_t)m);
    const uint32_t rem = (uint32_t)m - n * a.divPQ.d;
    const uint32_t p = a.divQ.div(rem);
    const uint32_t q = rem - p * a.divQ.d;
    const int ih = (int)p * a.stride + r - a.pad, iw = (int)q * a.stride + s - a.pad;
    if (ih < 0 || ih >= a.H || iw < 0 || iw >= a.W) return false;
    off = (((int64_t)n * a.H + ih) * a.W + iw) * a.C;
    return true;
  };

  auto gload = [&](int t) {
    const int mt = mbeg + t * DEPTH;
    if constexpr (F32) {
#pragma unroll
      for (int i = 0; i < A_CH32; ++i) {
        const int id = tid + i * 256, px = id / (BM / 4), kv = id % (BM / 4);
        const int m = mt + px;
        ra[i] = (px < DEPTH && m < mend) ? *reinterpret_cast<const Chunk*>(dz + (int64_t)m * a.K + k0 + kv * 4)
                                         : Chunk{{0u, 0u, 0u, 0u}};
      }
#pragma unroll
      for (int i = 0; i < B_CH32; ++i) {
        const int id = tid + i * 256, px = id / (BN / 4), cv = id % (BN / 4);
        int64_t off = 0;
        const bool ok = px < DEPTH && src_pixel(mt + px, off);
        rb[i] = ok ? *reinterpret_cast<const Chunk*>(x + off + c0 + cv * 4) : Chunk{{0u, 0u, 0u, 0u}};
      }
    } else {
      {
        const int cp = tid % (BM / 2), pg = tid / (BM / 2);
#pragma unroll
        for (int i = 0; i < PXA; ++i) {
          const int m = mt + pg * PXA + i;
          ha[i] = m < mend ? *reinterpret_cast<const uint32_t*>(dz + (int64_t)m * a.K + k0 + 2 * cp) : 0u;
        }
      }
      {
        const int cp = tid % (BN / 2), pg = tid / (BN / 2);
#pragma unroll
        for (int i = 0; i < PXB; ++i) {
          int64_t off = 0;
          const bool ok = src_pixel(mt + pg * PXB + i, off);
          hb[i] = ok ? *reinterpret_cast<const uint32_t*>(x + off + c0 + 2 * cp) : 0u;
        }
      }
    }
  };
  auto sstore = [&](int buf) {
    if constexpr (F32) {
#pragma unroll
      for (int i = 0; i < A_CH32; ++i) {
        const int id = tid + i * 256, px = id / (BM / 4), kv = id % (BM / 4);
        if (px < DEPTH) *reinterpret_cast<Chunk*>(&As[buf][px * (BM + 4) + kv * 4]) = ra[i];
      }
#pragma unroll
      for (int i = 0; i < B_CH32; ++i) {
        const int id = tid + i * 256, px = id / (BN / 4), cv = id % (BN / 4);
        if (px < DEPTH) *reinterpret_cast<Chunk*>(&Bs[buf][px * (BN + 4) + cv * 4]) = rb[i];
      }
    } else {
      {
        const int cp = tid % (BM / 2), pg = tid / (BM / 2);
        uint32_t* lo = reinterpret_cast<uint32_t*>(&As[buf][(2 * cp) * (DEPTH + 8) + pg * PXA]);
        uint32_t* hi = reinterpret_cast<uint32_t*>(&As[buf][(2 * cp + 1) * (DEPTH + 8) + pg * PXA]);
#pragma unroll
        for (int i = 0; i < PXA / 2; ++i) { lo[i] = pack_lo(ha[2 * i], ha[2 * i + 1]); hi[i] = pack_hi(ha[2 * i], ha[2 * i + 1]); }
      }
      {
        const int cp = tid % (BN / 2), pg = tid / (BN / 2);
        uint32_t* lo = reinterpret_cast<uint32_t*>(&Bs[buf][(2 * cp) * (DEPTH + 8) + pg * PXB]);
        uint32_t* hi = reinterpret_cast<uint32_t*>(&Bs[buf][(2 * cp + 1) * (DEPTH + 8) + pg * PXB]);
#pragma unroll
        for (int i = 0; i < PXB / 2; ++i) { lo[i] = pack_lo(hb[2 * i], hb[2 * i + 1]); hi[i] = pack_hi(hb[2 * i], hb[2 * i + 1]); }
      }
    }
  };

  v16f acc[MI][NI];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NI; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  if (ntiles > 0) {
    gload(0);
    sstore(0);
  }
  __syncthreads();
  for (int t = 0; t < ntiles; ++t) {
    const int buf = t & 1;
    if (t + 1 < ntiles) gload(t + 1);
    if constexpr (F32) {
      WFrag<float> fa[MI], fb[NI];
#pragma unroll
      for (int i = 0; i < MI; ++i) fa[i].load(reinterpret_cast<const float*>(As[buf]), BM + 4, wm * (BM / 2) + i * 32 + l32, g);
#pragma unroll
      for (int j = 0; j < NI; ++j) fb[j].load(reinterpret_cast<const float*>(Bs[buf]), BN + 4, wn * (BN / 2) + j * 32 + l32, g);
#pragma unroll
      for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j) WFrag<float>::mma(fa[i], fb[j], acc[i][j]);
    } else {
      Frag<T> fa[MI], fb[NI];
#pragma unroll
      for (int i = 0; i < MI; ++i) fa[i].load(&As[buf][(wm * (BM / 2) + i * 32 + l32) * (DEPTH + 8) + g * 16]);
#pragma unroll
      for (int j = 0; j < NI; ++j) fb[j].load(&Bs[buf][(wn * (BN / 2) + j * 32 + l32) * (DEPTH + 8) + g * 16]);
#pragma unroll
      for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j) Frag<T>::mma(fa[i], fb[j], acc[i][j]);
    }
    if (t + 1 < ntiles) sstore(buf ^ 1);
    __syncthreads();
  }

  const int64_t outputs = (int64_t)a.K * a.R * a.S * a.C;
  float* dst = out + (int64_t)blockIdx.z * outputs;
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NI; ++j) {
      const int c = c0 + wn * (BN / 2) + j * 32 + l32;
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int k = k0 + wm * (BM / 2) + i * 32 + 8 * (e >> 2) + 4 * g + (e & 3);
        dst[((int64_t)k * a.R * a.S + tap) * a.C + c] = acc[i][j][e];
      }
    }
}

bool conv_mfma_wgrad_ok(int dt, const ConvGeom& g) {
  (void)dt;
  return g.C % 64 == 0 && g.K % 64 == 0 && (int64_t)g.N * g.P * g.Q < (1 << 24) && g.P * g.Q < (1 << 24);
}

// number of pixel chunks, from the layer shape only
int conv_mfma_wgrad_splits(int dt, const ConvGeom& g) {
  const int depth = dt == DT_F32 ? 16 : 32;
  const int bm = g.K % 128 == 0 ? 128 : 64, bn = g.C % 128 == 0 ? 128 : 64;
  const int64_t tiles = (int64_t)(g.K / bm) * (g.C / bn) * g.R * g.S;
  const int64_t pixels = (int64_t)g.N * g.P * g.Q;
  int64_t want = (1024 + tiles - 1) / tiles;                       // aim at ~1024 blocks
  const int64_t most = (pixels + 4 * depth - 1) / (4 * depth);     // at least four depth tiles per chunk
  if (want > most) want = most;
  if (want > 64) want = 64;
  return (int)(want < 1 ? 1 : want);
}

template <class T>
static void launch_wgrad_t(hipStream_t st, const void* x, const void* dz, float* dst, int splits, const ConvGeom& g) {
  constexpr int depth = sizeof(T) == 4 ? 16 : 32;
  WGradArgs a;
  a.H = g.H; a.W = g.W; a.C = g.C; a.K = g.K; a.R = g.R; a.S = g.S; a.stride = g.stride; a.pad = g.pad; a.P = g.P; a.Q = g.Q;
  a.pixels = g.N * g.P * g.Q;
  int chunk = (a.pixels + splits - 1) / splits;
  a.chunk = (chunk + depth - 1) / depth * depth;
  a.divQ = make_fastdiv((uint32_t)g.Q);
  a.divPQ = make_fastdiv((uint32_t)(g.P * g.Q));
  const bool m128 = g.K % 128 == 0, n128 = g.C % 128 == 0;
  const int bm = m128 ? 128 : 64, bn = n128 ? 128 : 64;
  dim3 grid(g.K / bm, g.R * g.S * (g.C / bn), splits), block(256);
  if (m128 && n128) hipLaunchKernelGGL((conv_wgrad_kernel<T, 128, 128>), grid, block, 0, st, (const T*)x, (const T*)dz, dst, a);
  else if (m128) hipLaunchKernelGGL((conv_wgrad_kernel<T, 128, 64>), grid, block, 0, st, (const T*)x, (const T*)dz, dst, a);
  else if (n128) hipLaunchKernelGGL((conv_wgrad_kernel<T, 64, 128>), grid, block, 0, st, (const T*)x, (const T*)dz, dst, a);
  else hipLaunchKernelGGL((conv_wgrad_kernel<T, 64, 64>), grid, block, 0, st, (const T*)x, (const T*)dz, dst, a);
}

__global__ void wgrad_reduce_kernel(const float* __restrict__ partial, float* __restrict__ out, int64_t n, int splits) {
  const int64_t i = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) * 4;
  if (i >= n) return;
  v4f acc = *reinterpret_cast<const v4f*>(partial + i);
  for (int s = 1; s < splits; ++s) acc += *reinterpret_cast<const v4f*>(partial + (int64_t)s * n + i);
  *reinterpret_cast<v4f*>(out + i) = acc;
}

void launch_conv_wgrad_mfma(hipStream_t st, int dt, const void* x, const void* dz, float* dw, float* partial, int splits,
                            const ConvGeom& g) {
  float* dst = splits > 1 ? partial : dw;
  if (dt == DT_F32) launch_wgrad_t<float>(st, x, dz, dst, splits, g);
  else if (dt == DT_BF16) launch_wgrad_t<bf16_t>(st, x, dz, dst, splits, g);
  else launch_wgrad_t<f16_t>(st, x, dz, dst, splits, g);
  if (splits > 1) {
    const int64_t n = (int64_t)g.K * g.R * g.S * g.C;  // a multiple of 4 (C % 64 == 0)
    hipLaunchKernelGGL(wgrad_reduce_kernel, dim3(ceil_div(n / 4, 256)), dim3(256), 0, st, partial, dw, n, splits);
  }
}

}  // namespace oseq
