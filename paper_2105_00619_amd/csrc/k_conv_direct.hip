// Direct (plain FMA) convolution forward / data gradient / weight gradient for shapes the matrix-core
// kernels do not take: very few channels (the 3-channel stem, the tiny test networks).  NHWC activations,
// (C_out, kh, kw, C_in) weights, fp32 accumulation in a fixed order.
#include "dev_common.h"
#include "kernels.h"

namespace oseq {

template <class T>
__global__ void __launch_bounds__(256) conv_fwd_direct_kernel(const T* __restrict__ x, const T* __restrict__ w,
                                                              const float* __restrict__ bias, T* __restrict__ out,
                                                              ConvGeom g, int relu) {
  const int64_t total = (int64_t)g.N * g.P * g.Q * g.K;
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= total) return;
  const int k = (int)(i % g.K);
  int64_t t = i / g.K;
  const int q = (int)(t % g.Q); t /= g.Q;
  const int p = (int)(t % g.P);
  const int n = (int)(t / g.P);
  float acc = 0.f;
  for (int r = 0; r < g.R; ++r) {
    const int ih = p * g.stride + r - g.pad;
    if (ih < 0 || ih >= g.H) continue;
    for (int s = 0; s < g.S; ++s) {
      const int iw = q * g.stride + s - g.pad;
      if (iw < 0 || iw >= g.W) continue;
      const T* xp = x + (((int64_t)n * g.H + ih) * g.W + iw) * g.C;
      const T* wp = w + (((int64_t)k * g.R + r) * g.S + s) * g.C;
      for (int c = 0; c < g.C; ++c) acc = __fmaf_rn(to_f32(xp[c]), to_f32(wp[c]), acc);
    }
  }
  if (bias) acc += bias[k];
  if (relu) acc = fmaxf(acc, 0.f);
  out[i] = from_f32<T>(acc);
}

// dx[n,h,w,c] = sum_{r,s,k} dz[n,p,q,k] * w[k,r,s,c] over the (p,q) with p*stride + r - pad == h, q*stride + s - pad == w
template <class T>
__global__ void __launch_bounds__(256) conv_dgrad_direct_kernel(const T* __restrict__ dz, const T* __restrict__ w,
                                                                const T* __restrict__ addend, T* __restrict__ dx,
                                                                ConvGeom g) {
  const int64_t total = (int64_t)g.N * g.H * g.W * g.C;
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= total) return;
  const int c = (int)(i % g.C);
  int64_t t = i / g.C;
  const int wq = (int)(t % g.W); t /= g.W;
  const int h = (int)(t % g.H);
  const int n = (int)(t / g.H);
  float acc = 0.f;
  for (int r = 0; r < g.R; ++r) {
    const int ph = h + g.pad - r;
    if (ph < 0 || ph % g.stride) continue;
    const int p = ph / g.stride;
    if (p >= g.P) continue;
    for (int s = 0; s < g.S; ++s) {
      const int qw = wq + g.pad - s;
      if (qw < 0 || qw % g.stride) continue;
      const int q = qw / g.stride;
      if (q >= g.Q) continue;
      const T* zp = dz + (((int64_t)n * g.P + p) * g.Q + q) * g.K;
      const T* wp = w + ((int64_t)r * g.S + s) * g.C + c;
      const int64_t wk = (int64_t)g.R * g.S * g.C;
      for (int k = 0; k < g.K; ++k) acc = __fmaf_rn(to_f32(zp[k]), to_f32(wp[k * wk]), acc);
    }
  }
  if (addend) acc += to_f32(addend[i]);
  dx[i] = from_f32<T>(acc);
}

// dw[k,r,s,c] = sum over pixels (n,p,q) of dz[n,p,q,k] * x[n, p*stride+r-pad, q*stride+s-pad, c];
// blockIdx.y selects a fixed chunk of the pixel range; chunks are summed afterwards in order.
template <class T>
__global__ void __launch_bounds__(256) conv_wgrad_direct_kernel(const T* __restrict__ x, const T* __restrict__ dz,
                                                                float* __restrict__ out, ConvGeom g, int64_t chunk) {
  const int64_t outputs = (int64_t)g.K * g.R * g.S * g.C;
  const int64_t o = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (o >= outputs) return;
  const int c = (int)(o % g.C);
  int64_t t = o / g.C;
  const int s = (int)(t % g.S); t /= g.S;
  const int r = (int)(t % g.R);
  const int k = (int)(t / g.R);
  const int64_t pixels = (int64_t)g.N * g.P * g.Q;
  const int64_t m0 = (int64_t)blockIdx.y * chunk;
  const int64_t m1 = m0 + chunk < pixels ? m0 + chunk : pixels;
  float acc = 0.f;
  for (int64_t m = m0; m < m1; ++m) {
    const int q = (int)(m % g.Q);
    const int64_t u = m / g.Q;
    const int p = (int)(u % g.P);
    const int n = (int)(u / g.P);
    const int ih = p * g.stride + r - g.pad, iw = q * g.stride + s - g.pad;
    if (ih < 0 || ih >= g.H || iw < 0 || iw >= g.W) continue;
    acc = __fmaf_rn(to_f32(dz[m * g.K + k]), to_f32(x[(((int64_t)n * g.H + ih) * g.W + iw) * g.C + c]), acc);
  }
  out[(int64_t)blockIdx.y * outputs + o] = acc;
}

__global__ void splitk_reduce_kernel(const float* __restrict__ partial, float* __restrict__ out, int64_t n, int splits) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  float acc = 0.f;
  for (int s = 0; s < splits; ++s) acc += partial[(int64_t)s * n + i];
  out[i] = acc;
}

// ------------------------------------------------------------------------------------------------------------
// Few input channels (the 3-channel stem): R*S*C <= 36 products per output.  HBM-bound (one activation write per
// 27 multiply-adds per channel), so plain FMAs: a thread keeps its pixel's input patch in registers and produces
// 8 output channels; the 8 x (R*S*C) weights of the block's channel group sit in LDS and are read by broadcast.
// ------------------------------------------------------------------------------------------------------------
constexpr int SMALLC_MAX = 36;

template <class T, int C>
__global__ void __launch_bounds__(256) conv_fwd_smallc_kernel(const T* __restrict__ x, const T* __restrict__ w,
                                                              const float* __restrict__ bias, T* __restrict__ out,
                                                              ConvGeom g, int relu) {
  constexpr int RSC = 9 * C;  // 3x3 filter
  __shared__ float ws[8 * RSC];
  const int kg = blockIdx.y;
  for (int i = threadIdx.x; i < 8 * RSC; i += 256) ws[i] = to_f32(w[(int64_t)kg * 8 * RSC + i]);
  __syncthreads();
  const int64_t m = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (m >= (int64_t)g.N * g.P * g.Q) return;
  const int q = (int)(m % g.Q);
  const int64_t t = m / g.Q;
  const int p = (int)(t % g.P), n = (int)(t / g.P);
  float xin[RSC];
#pragma unroll
  for (int r = 0; r < 3; ++r) {
    const int ih = p * g.stride + r - g.pad;
#pragma unroll
    for (int s = 0; s < 3; ++s) {
      const int iw = q * g.stride + s - g.pad;
      const bool ok = ih >= 0 && ih < g.H && iw >= 0 && iw < g.W;
      const T* xp = x + (((int64_t)n * g.H + (ok ? ih : 0)) * g.W + (ok ? iw : 0)) * C;
#pragma unroll
      for (int c = 0; c < C; ++c) xin[(r * 3 + s) * C + c] = ok ? to_f32(xp[c]) : 0.f;
    }
  }
  float acc[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    float a = 0.f;
#pragma unroll
    for (int i = 0; i < RSC; ++i) a = __fmaf_rn(xin[i], ws[j * RSC + i], a);
    if (bias) a += bias[kg * 8 + j];
    acc[j] = relu ? fmaxf(a, 0.f) : a;
  }
  store_f32<T, 8>(out + m * g.K + kg * 8, acc);
}

// weight gradient for few input channels: a block reduces a fixed chunk of pixels; thread (k, ti) accumulates
// dw[k][i] for i = ti, ti+4, ...; dz and the input patches of 64 pixels at a time are staged in LDS as fp32
template <class T>
__global__ void __launch_bounds__(256) conv_wgrad_smallc_kernel(const T* __restrict__ x, const T* __restrict__ dz,
                                                                float* __restrict__ partial, ConvGeom g, int chunk) {
  __shared__ float dzs[64 * 65];
  __shared__ float xs[64 * (SMALLC_MAX + 1)];
  const int rsc = g.R * g.S * g.C;
  const int tk = threadIdx.x & 63, ti = threadIdx.x >> 6;
  const int64_t pixels = (int64_t)g.N * g.P * g.Q;
  const int64_t m0 = (int64_t)blockIdx.x * chunk;
  const int64_t m1 = m0 + chunk < pixels ? m0 + chunk : pixels;
  float acc[SMALLC_MAX / 4];
#pragma unroll
  for (int j = 0; j < SMALLC_MAX / 4; ++j) acc[j] = 0.f;
  for (int64_t mt = m0; mt < m1; mt += 64) {
    // all global loads of the sub-tile are issued before the first LDS store (fixed trip counts, unrolled)
    float vd[16], vx[(64 * SMALLC_MAX + 255) / 256];
#pragma unroll
    for (int it = 0; it < 16; ++it) {
      const int i = threadIdx.x + it * 256;
      const int px = i / g.K, k = i - px * g.K;
      vd[it] = (i < 64 * g.K && mt + px < m1) ? to_f32(dz[(mt + px) * g.K + k]) : 0.f;
    }
#pragma unroll
    for (int it = 0; it < (64 * SMALLC_MAX + 255) / 256; ++it) {
      const int i = threadIdx.x + it * 256;
      const int px = i / rsc, e = i - px * rsc;
      float v = 0.f;
      const int64_t m = mt + px;
      if (i < 64 * rsc && m < m1) {
        const int c = e % g.C, tap = e / g.C, s = tap % g.S, r = tap / g.S;
        const int q = (int)(m % g.Q);
        const int64_t t = m / g.Q;
        const int p = (int)(t % g.P), n = (int)(t / g.P);
        const int ih = p * g.stride + r - g.pad, iw = q * g.stride + s - g.pad;
        if (ih >= 0 && ih < g.H && iw >= 0 && iw < g.W) v = to_f32(x[(((int64_t)n * g.H + ih) * g.W + iw) * g.C + c]);
      }
      vx[it] = v;
    }
#pragma unroll
    for (int it = 0; it < 16; ++it) {
      const int i = threadIdx.x + it * 256;
      const int px = i / g.K, k = i - px * g.K;
      if (i < 64 * g.K) dzs[px * 65 + k] = vd[it];
    }
#pragma unroll
    for (int it = 0; it < (64 * SMALLC_MAX + 255) / 256; ++it) {
      const int i = threadIdx.x + it * 256;
      const int px = i / rsc, e = i - px * rsc;
      if (i < 64 * rsc) xs[px * (SMALLC_MAX + 1) + e] = vx[it];
    }
    __syncthreads();
    if (tk < g.K) {
#pragma unroll 4
      for (int px = 0; px < 64; ++px) {
        const float d = dzs[px * 65 + tk];
#pragma unroll
        for (int j = 0; j < SMALLC_MAX / 4; ++j)
          if (ti + 4 * j < rsc) acc[j] = __fmaf_rn(d, xs[px * (SMALLC_MAX + 1) + ti + 4 * j], acc[j]);
      }
    }
    __syncthreads();
  }
  if (tk < g.K) {
#pragma unroll
    for (int j = 0; j < SMALLC_MAX / 4; ++j)
      if (ti + 4 * j < rsc) partial[((int64_t)blockIdx.x * g.K + tk) * rsc + ti + 4 * j] = acc[j];
  }
}

// one wavefront per output: lanes sum the block partials l, l+64, ... then a fixed butterfly
__global__ void __launch_bounds__(256) wave_reduce_kernel(const float* __restrict__ partial, float* __restrict__ out, int64_t n,
                                                          int splits) {
  const int64_t o = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (o >= n) return;
  float v = 0.f;
  for (int s = threadIdx.x & 63; s < splits; s += 64) v += partial[(int64_t)s * n + o];
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  if ((threadIdx.x & 63) == 0) out[o] = v;
}

bool conv_smallc_fwd_ok(const ConvGeom& g) { return g.C <= 4 && g.R == 3 && g.S == 3 && g.K % 8 == 0; }
bool conv_smallc_wgrad_ok(const ConvGeom& g) { return g.C <= 4 && g.R * g.S * g.C <= SMALLC_MAX && g.K <= 64; }
int conv_smallc_wgrad_splits(const ConvGeom& g) {
  const int64_t pixels = (int64_t)g.N * g.P * g.Q;
  int64_t b = (pixels + 255) / 256;
  return (int)(b < 1 ? 1 : (b > 1024 ? 1024 : b));
}

template <class T>
static void launch_fwd_smallc_t(hipStream_t st, const void* x, const void* w, const float* bias, void* out, const ConvGeom& g,
                                int relu) {
  dim3 grid(ceil_div((int64_t)g.N * g.P * g.Q, 256), g.K / 8), block(256);
  switch (g.C) {
    case 1: hipLaunchKernelGGL((conv_fwd_smallc_kernel<T, 1>), grid, block, 0, st, (const T*)x, (const T*)w, bias, (T*)out, g, relu); break;
    case 2: hipLaunchKernelGGL((conv_fwd_smallc_kernel<T, 2>), grid, block, 0, st, (const T*)x, (const T*)w, bias, (T*)out, g, relu); break;
    case 3: hipLaunchKernelGGL((conv_fwd_smallc_kernel<T, 3>), grid, block, 0, st, (const T*)x, (const T*)w, bias, (T*)out, g, relu); break;
    default: hipLaunchKernelGGL((conv_fwd_smallc_kernel<T, 4>), grid, block, 0, st, (const T*)x, (const T*)w, bias, (T*)out, g, relu); break;
  }
}

void launch_conv_fwd_smallc(hipStream_t st, int dt, const void* x, const void* w, const float* bias, void* out,
                            const ConvGeom& g, int relu) {
  if (dt == DT_F32) launch_fwd_smallc_t<float>(st, x, w, bias, out, g, relu);
  else if (dt == DT_BF16) launch_fwd_smallc_t<bf16_t>(st, x, w, bias, out, g, relu);
  else launch_fwd_smallc_t<f16_t>(st, x, w, bias, out, g, relu);
}

// partial: [splits][K][R*S*C] floats; splits = conv_smallc_wgrad_splits(g)
void launch_conv_wgrad_smallc(hipStream_t st, int dt, const void* x, const void* dz, float* dw, float* partial, int splits,
                              const ConvGeom& g) {
  const int64_t pixels = (int64_t)g.N * g.P * g.Q;
  int chunk = (int)((pixels + splits - 1) / splits);
  chunk = (chunk + 63) / 64 * 64;
  float* dst = splits > 1 ? partial : dw;
  dim3 grid(splits), block(256);
  if (dt == DT_F32) hipLaunchKernelGGL(conv_wgrad_smallc_kernel<float>, grid, block, 0, st, (const float*)x, (const float*)dz, dst, g, chunk);
  else if (dt == DT_BF16) hipLaunchKernelGGL(conv_wgrad_smallc_kernel<bf16_t>, grid, block, 0, st, (const bf16_t*)x, (const bf16_t*)dz, dst, g, chunk);
  else hipLaunchKernelGGL(conv_wgrad_smallc_kernel<f16_t>, grid, block, 0, st, (const f16_t*)x, (const f16_t*)dz, dst, g, chunk);
  if (splits > 1) {
    const int64_t n = (int64_t)g.K * g.R * g.S * g.C;
    hipLaunchKernelGGL(wave_reduce_kernel, dim3(ceil_div(n, 4)), dim3(256), 0, st, partial, dw, n, splits);
  }
}

void launch_conv_fwd_direct(hipStream_t st, int dt, const void* x, const void* w, const float* bias, void* out,
                            const ConvGeom& g, int relu) {
  const int64_t total = (int64_t)g.N * g.P * g.Q * g.K;
  dim3 grid(ceil_div(total, 256)), block(256);
  if (dt == DT_F32) hipLaunchKernelGGL(conv_fwd_direct_kernel<float>, grid, block, 0, st, (const float*)x, (const float*)w, bias, (float*)out, g, relu);
  else if (dt == DT_BF16) hipLaunchKernelGGL(conv_fwd_direct_kernel<bf16_t>, grid, block, 0, st, (const bf16_t*)x, (const bf16_t*)w, bias, (bf16_t*)out, g, relu);
  else hipLaunchKernelGGL(conv_fwd_direct_kernel<f16_t>, grid, block, 0, st, (const f16_t*)x, (const f16_t*)w, bias, (f16_t*)out, g, relu);
}

void launch_conv_dgrad_direct(hipStream_t st, int dt, const void* dz, const void* w, const void* addend, void* dx,
                              const ConvGeom& g) {
  const int64_t total = (int64_t)g.N * g.H * g.W * g.C;
  dim3 grid(ceil_div(total, 256)), block(256);
  if (dt == DT_F32) hipLaunchKernelGGL(conv_dgrad_direct_kernel<float>, grid, block, 0, st, (const float*)dz, (const float*)w, (const float*)addend, (float*)dx, g);
  else if (dt == DT_BF16) hipLaunchKernelGGL(conv_dgrad_direct_kernel<bf16_t>, grid, block, 0, st, (const bf16_t*)dz, (const bf16_t*)w, (const bf16_t*)addend, (bf16_t*)dx, g);
  else hipLaunchKernelGGL(conv_dgrad_direct_kernel<f16_t>, grid, block, 0, st, (const f16_t*)dz, (const f16_t*)w, (const f16_t*)addend, (f16_t*)dx, g);
}

void launch_conv_wgrad_direct(hipStream_t st, int dt, const void* x, const void* dz, float* dw, float* partial, int splits,
                              const ConvGeom& g) {
  const int64_t outputs = (int64_t)g.K * g.R * g.S * g.C;
  const int64_t pixels = (int64_t)g.N * g.P * g.Q;
  const int64_t chunk = (pixels + splits - 1) / splits;
  float* dst = splits > 1 ? partial : dw;
  dim3 grid(ceil_div(outputs, 256), splits), block(256);
  if (dt == DT_F32) hipLaunchKernelGGL(conv_wgrad_direct_kernel<float>, grid, block, 0, st, (const float*)x, (const float*)dz, dst, g, chunk);
  else if (dt == DT_BF16) hipLaunchKernelGGL(conv_wgrad_direct_kernel<bf16_t>, grid, block, 0, st, (const bf16_t*)x, (const bf16_t*)dz, dst, g, chunk);
  else hipLaunchKernelGGL(conv_wgrad_direct_kernel<f16_t>, grid, block, 0, st, (const f16_t*)x, (const f16_t*)dz, dst, g, chunk);
  if (splits > 1)
    hipLaunchKernelGGL(splitk_reduce_kernel, dim3(ceil_div(outputs, 256)), dim3(256), 0, st, partial, dw, outputs, splits);
}

}  // namespace oseq
