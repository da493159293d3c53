// Fused mixed-precision optimizer step over the flat parameter arena (Section "Mixed-precision training":
// 32-bit master weights and update, 16-bit copies for the next forward pass):
//   pass 1: found_inf = any gradient not finite
//   pass 2: if !found_inf:  g <- g / S ;  v <- mu*v + g ;  w <- w - lr*v ;  w16 <- cast(w)
// Pass 2 reads the flag on the device, so a skipped step costs no host round trip.
#include "dev_common.h"
#include "kernels.h"

namespace oseq {

// Clears the step's flags and validates the labels before anything else runs: flags[0] = a gradient is not finite
// (set by the check pass), flags[1] = a label lies outside [0, classes).  Either flag makes the update pass a no-op,
// and flags[1] also keeps the BatchNorm running statistics as they were.  One block; stream order makes the flags
// visible to every later kernel of the step.
__global__ void __launch_bounds__(256) step_init_kernel(int* __restrict__ flags, const int32_t* __restrict__ y, int n,
                                                        int classes) {
  __shared__ int bad;
  if (threadIdx.x == 0) bad = 0;
  __syncthreads();
  bool b = false;
  for (int i = threadIdx.x; i < n; i += blockDim.x) b |= y[i] < 0 || y[i] >= classes;
  if (b) bad = 1;  // every writer stores the same value
  __syncthreads();
  if (threadIdx.x < 4) flags[threadIdx.x] = threadIdx.x == 1 ? bad : 0;
}

typedef __attribute__((ext_vector_type(4))) float opt_v4f;

// Both passes handle four consecutive parameters per thread and trip (16-byte accesses; the arrays start on 256-byte
// boundaries), all loads of a trip before its stores; the last n % 4 parameters are handled by the first threads.
__global__ void __launch_bounds__(256) optim_check_kernel(const float* __restrict__ g, int64_t n, int* __restrict__ flags) {
  const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  const int64_t n4 = n / 4;
  bool bad = false;
  for (int64_t i = t; i < n4; i += stride) {
    const opt_v4f v = *reinterpret_cast<const opt_v4f*>(g + 4 * i);
#pragma unroll
    for (int e = 0; e < 4; ++e) bad |= (__float_as_uint(v[e]) & 0x7f800000u) == 0x7f800000u;
  }
  if (t < n - 4 * n4) bad |= (__float_as_uint(g[4 * n4 + t]) & 0x7f800000u) == 0x7f800000u;
  if (__any(bad) && (threadIdx.x & 63) == 0) atomicOr(flags, 1);
}

template <class T, bool HALF>
__global__ void __launch_bounds__(256) optim_update_kernel(float* __restrict__ w, float* __restrict__ v,
                                                           const float* __restrict__ g, T* __restrict__ w16,
                                                           float* __restrict__ gout, int64_t n, float lr, float mom,
                                                           float inv_scale, const int* __restrict__ flags) {
  if (flags[0] | flags[1]) return;  // non-finite gradient or invalid label: the step changes nothing
  const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  const int64_t n4 = n / 4;
  const bool gout_aligned = (reinterpret_cast<uintptr_t>(gout) & 15) == 0;
  auto one = [&](float gi_scaled, float wi, float vi_in, float& vi_out) {
    if (mom != 0.f) {
      vi_out = __fmaf_rn(mom, vi_in, gi_scaled);
      return wi - lr * vi_out;
    }
    vi_out = vi_in;
    return wi - lr * gi_scaled;
  };
  for (int64_t i = t; i < n4; i += stride) {
    const opt_v4f gv = *reinterpret_cast<const opt_v4f*>(g + 4 * i);
    const opt_v4f wv = *reinterpret_cast<const opt_v4f*>(w + 4 * i);
    opt_v4f vv = {0.f, 0.f, 0.f, 0.f};
    if (mom != 0.f) vv = *reinterpret_cast<const opt_v4f*>(v + 4 * i);
    opt_v4f gs, wn, vn;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      gs[e] = gv[e] * inv_scale;
      float vo;
      wn[e] = one(gs[e], wv[e], vv[e], vo);
      vn[e] = vo;
    }
    if (mom != 0.f) *reinterpret_cast<opt_v4f*>(v + 4 * i) = vn;
    *reinterpret_cast<opt_v4f*>(w + 4 * i) = wn;
    if (HALF) {
      float h[4] = {wn[0], wn[1], wn[2], wn[3]};
      store_f32<T, 4>(w16 + 4 * i, h);
    }
    if (gout) {  // the caller's buffer: 16-byte stores only if it is aligned for them
      if (gout_aligned) *reinterpret_cast<opt_v4f*>(gout + 4 * i) = gs;
      else { gout[4 * i] = gs[0]; gout[4 * i + 1] = gs[1]; gout[4 * i + 2] = gs[2]; gout[4 * i + 3] = gs[3]; }
    }
  }
  if (t < n - 4 * n4) {
    const int64_t i = 4 * n4 + t;
    const float gi = g[i] * inv_scale;
    float vo;
    const float wi = one(gi, w[i], mom != 0.f ? v[i] : 0.f, vo);
    if (mom != 0.f) v[i] = vo;
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
// four parameters per thread and trip
static int grid4_for(int64_t n) { return grid_for((n + 3) / 4); }

void launch_step_init(hipStream_t st, int* flags, const int32_t* y, int n, int classes) {
  OSEQ_LAUNCH(step_init_kernel, dim3(1), dim3(256), 0, st, flags, y, n, classes);
}

void launch_optim(hipStream_t st, int dt, float* w, float* v, const float* g, void* w16, float* gout, int64_t n, float lr,
                  float mom, float inv_scale, int* flags) {
  OSEQ_LAUNCH(optim_check_kernel, dim3(grid4_for(n)), dim3(256), 0, st, g, n, flags);
  if (dt == DT_F32) OSEQ_LAUNCH((optim_update_kernel<float, false>), dim3(grid4_for(n)), dim3(256), 0, st, w, v, g, (float*)nullptr, gout, n, lr, mom, inv_scale, flags);
  else if (dt == DT_BF16) OSEQ_LAUNCH((optim_update_kernel<bf16_t, true>), dim3(grid4_for(n)), dim3(256), 0, st, w, v, g, (bf16_t*)w16, gout, n, lr, mom, inv_scale, flags);
  else OSEQ_LAUNCH((optim_update_kernel<f16_t, true>), dim3(grid4_for(n)), dim3(256), 0, st, w, v, g, (f16_t*)w16, gout, n, lr, mom, inv_scale, flags);
}

void launch_cast_params(hipStream_t st, int dt, const float* w, void* w16, int64_t n) {
  if (dt == DT_BF16) OSEQ_LAUNCH(cast_params_kernel<bf16_t>, dim3(grid_for(n)), dim3(256), 0, st, w, (bf16_t*)w16, n);
  else if (dt == DT_F16) OSEQ_LAUNCH(cast_params_kernel<f16_t>, dim3(grid_for(n)), dim3(256), 0, st, w, (f16_t*)w16, n);
}

void launch_fill(hipStream_t st, float* p, int64_t n, float v) {
  if (n > 0) OSEQ_LAUNCH(fill_kernel, dim3(grid_for(n)), dim3(256), 0, st, p, n, v);
}

}  // namespace oseq
