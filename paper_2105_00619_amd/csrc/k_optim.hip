// Fused mixed-precision optimizer step over the flat parameter arena (Section "Mixed-precision training":
// 32-bit master weights and update, 16-bit copies for the next forward pass):
//   pass 1: found_inf = any gradient not finite
//   pass 2: if !found_inf:  g <- g / S ;  v <- mu*v + g ;  w <- w - lr*v ;  w16 <- cast(w)
// Pass 2 reads the flag on the device, so a skipped step costs no host round trip.
#include "dev_common.h"
#include "kernels.h"

namespace oseq {

__global__ void step_init_kernel(int* flags) {
  if (threadIdx.x < 4) flags[threadIdx.x] = 0;
}

__global__ void __launch_bounds__(256) optim_check_kernel(const float* __restrict__ g, int64_t n, int* __restrict__ flags) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  bool bad = false;
  for (; i < n; i += stride) {
    const uint32_t u = __float_as_uint(g[i]);
    bad |= (u & 0x7f800000u) == 0x7f800000u;
  }
  if (__any(bad) && (threadIdx.x & 63) == 0) atomicOr(flags, 1);
}

template <class T, bool HALF>
__global__ void __launch_bounds__(256) optim_update_kernel(float* __restrict__ w, float* __restrict__ v,
                                                           const float* __restrict__ g, T* __restrict__ w16,
                                                           float* __restrict__ gout, int64_t n, float lr, float mom,
                                                           float inv_scale, const int* __restrict__ flags) {
  if (flags[0]) return;
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) {
    const float gi = g[i] * inv_scale;
    float wi = w[i];
    if (mom != 0.f) {
      const float vi = __fmaf_rn(mom, v[i], gi);
      v[i] = vi;
      wi = wi - lr * vi;
    } else {
      wi = wi - lr * gi;
    }
    w[i] = wi;
    if (HALF) w16[i] = from_f32<T>(wi);
    if (gout) gout[i] = gi;
  }
}

template <class T>
__global__ void cast_params_kernel(const float* __restrict__ w, T* __restrict__ w16, int64_t n) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) w16[i] = from_f32<T>(w[i]);
}

__global__ void fill_kernel(float* p, int64_t n, float v) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) p[i] = v;
}

static int grid_for(int64_t n) { int64_t b = (n + 255) / 256; return (int)(b < 1 ? 1 : (b > 8192 ? 8192 : b)); }

void launch_step_init(hipStream_t st, int* flags) { OSEQ_LAUNCH(step_init_kernel, dim3(1), dim3(64), 0, st, flags); }

void launch_optim(hipStream_t st, int dt, float* w, float* v, const float* g, void* w16, float* gout, int64_t n, float lr,
                  float mom, float inv_scale, int* flags) {
  OSEQ_LAUNCH(optim_check_kernel, dim3(grid_for(n)), dim3(256), 0, st, g, n, flags);
  if (dt == DT_F32) OSEQ_LAUNCH((optim_update_kernel<float, false>), dim3(grid_for(n)), dim3(256), 0, st, w, v, g, (float*)nullptr, gout, n, lr, mom, inv_scale, flags);
  else if (dt == DT_BF16) OSEQ_LAUNCH((optim_update_kernel<bf16_t, true>), dim3(grid_for(n)), dim3(256), 0, st, w, v, g, (bf16_t*)w16, gout, n, lr, mom, inv_scale, flags);
  else OSEQ_LAUNCH((optim_update_kernel<f16_t, true>), dim3(grid_for(n)), dim3(256), 0, st, w, v, g, (f16_t*)w16, gout, n, lr, mom, inv_scale, flags);
}

void launch_cast_params(hipStream_t st, int dt, const float* w, void* w16, int64_t n) {
  if (dt == DT_BF16) OSEQ_LAUNCH(cast_params_kernel<bf16_t>, dim3(grid_for(n)), dim3(256), 0, st, w, (bf16_t*)w16, n);
  else if (dt == DT_F16) OSEQ_LAUNCH(cast_params_kernel<f16_t>, dim3(grid_for(n)), dim3(256), 0, st, w, (f16_t*)w16, n);
}

void launch_fill(hipStream_t st, float* p, int64_t n, float v) {
  if (n > 0) OSEQ_LAUNCH(fill_kernel, dim3(grid_for(n)), dim3(256), 0, st, p, n, v);
}

}  // namespace oseq
