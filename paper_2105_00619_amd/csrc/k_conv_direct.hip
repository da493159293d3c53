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
