// Loss head: global average pool / flatten, linear layer, mean softmax cross-entropy, and their backward.
// All arithmetic in fp32 on fp32 master weights (the head is a few MFLOP; it is kept out of the 16-bit path
// for stability, in line with keeping loss computation in single precision).  Every sum runs in a fixed order.
#include "dev_common.h"
#include "kernels.h"

namespace oseq {

// feat[n][f]: GAP -> mean over H*W of channel f ; flatten -> x[n][f]
// GAP: block (n, g) owns 64 channels of image n; its four wavefronts take every fourth pixel (eight loads in flight
// per lane) and their sums are added in wavefront order.
template <class T>
__global__ void __launch_bounds__(256) head_feat_kernel(const T* __restrict__ x, float* __restrict__ feat, int HW, int C,
                                                        int gap) {
  __shared__ float sm[4][64];
  const int n = blockIdx.x;
  if (!gap) {
    const int64_t F = (int64_t)HW * C;
    for (int64_t i = (int64_t)blockIdx.y * 256 + threadIdx.x; i < F; i += (int64_t)gridDim.y * 256)
      feat[n * F + i] = to_f32(x[n * F + i]);
    return;
  }
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
  const int c = blockIdx.y * 64 + tx;
  float s = 0.f;
  if (c < C) {
    const T* col = x + (int64_t)n * HW * C + c;
#pragma unroll 8
    for (int p = ty; p < HW; p += 4) s += to_f32(col[(int64_t)p * C]);
  }
  sm[ty][tx] = s;
  __syncthreads();
  if (ty == 0 && c < C) feat[(int64_t)n * C + c] = (((sm[0][tx] + sm[1][tx]) + sm[2][tx]) + sm[3][tx]) / (float)HW;
}

// logits[n][j] = b[j] + sum_f feat[n][f] * w[j][f]: lanes stride over the features, then a fixed butterfly, per (sample,
// class).  A wavefront owns 8 samples x 8 classes, so that every feature and weight value it loads serves eight sums
// (one wavefront per (sample, class) re-read the whole weight matrix per sample: 508 us at batch 4096, 2048 features).
// With few samples the tiles are too few to fill the chip: then a wavefront keeps to one (sample, class).
template <int LIN_TN, int LIN_TJ>
__global__ void __launch_bounds__(256) linear_fwd_kernel(const float* __restrict__ feat, const float* __restrict__ w,
                                                         const float* __restrict__ b, float* __restrict__ logits, int N, int F,
                                                         int J) {
  const int jt = (J + LIN_TJ - 1) / LIN_TJ;
  const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int n0 = (t / jt) * LIN_TN, j0 = (t % jt) * LIN_TJ, lane = threadIdx.x & 63;
  if (n0 >= N) return;
  const float* fp[LIN_TN];
  const float* wp[LIN_TJ];
#pragma unroll
  for (int s = 0; s < LIN_TN; ++s) fp[s] = feat + (int64_t)(n0 + s < N ? n0 + s : n0) * F;
#pragma unroll
  for (int c = 0; c < LIN_TJ; ++c) wp[c] = w + (int64_t)(j0 + c < J ? j0 + c : j0) * F;
  float acc[LIN_TN][LIN_TJ];
#pragma unroll
  for (int s = 0; s < LIN_TN; ++s)
#pragma unroll
    for (int c = 0; c < LIN_TJ; ++c) acc[s][c] = 0.f;
  for (int f = lane; f < F; f += 64) {
    float x[LIN_TN], v[LIN_TJ];
#pragma unroll
    for (int s = 0; s < LIN_TN; ++s) x[s] = fp[s][f];
#pragma unroll
    for (int c = 0; c < LIN_TJ; ++c) v[c] = wp[c][f];
#pragma unroll
    for (int s = 0; s < LIN_TN; ++s)
#pragma unroll
      for (int c = 0; c < LIN_TJ; ++c) acc[s][c] = __fmaf_rn(x[s], v[c], acc[s][c]);
  }
#pragma unroll
  for (int s = 0; s < LIN_TN; ++s)
#pragma unroll
    for (int c = 0; c < LIN_TJ; ++c) {
      float a = acc[s][c];
#pragma unroll
      for (int off = 32; off > 0; off >>= 1) a += __shfl_xor(a, off, 64);
      if (lane == 0 && n0 + s < N && j0 + c < J) logits[(int64_t)(n0 + s) * J + j0 + c] = a + b[j0 + c];
    }
}

// per sample: loss_n = logsumexp(logits_n) - logits_n[y_n]; dlogits = (softmax - onehot) * gscale
// one wavefront per sample; lanes stride over the classes, maxima and sums by a fixed butterfly
__global__ void __launch_bounds__(256) softmax_ce_kernel(const float* __restrict__ logits, const int32_t* __restrict__ y,
                                                         float* __restrict__ loss_n, float* __restrict__ dlogits, int N, int J,
                                                         float gscale, int* __restrict__ flags) {
  const int n = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (n >= N) return;
  const int lane = threadIdx.x & 63;
  const float* lp = logits + (int64_t)n * J;
  float mx = -INFINITY;
  for (int j = lane; j < J; j += 64) mx = fmaxf(mx, lp[j]);
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off, 64));
  float se = 0.f;
  for (int j = lane; j < J; j += 64) se += expf(lp[j] - mx);
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) se += __shfl_xor(se, off, 64);
  const float lse = mx + logf(se);
  int lab = y[n];
  if (lab < 0 || lab >= J) { if (lane == 0) atomicOr(flags + 1, 1); lab = 0; }
  if (lane == 0) loss_n[n] = lse - lp[lab];
  const float inv = 1.f / se;
  for (int j = lane; j < J; j += 64) {
    const float pj = expf(lp[j] - mx) * inv;
    dlogits[(int64_t)n * J + j] = (pj - (j == lab ? 1.f : 0.f)) * gscale;
  }
}

__global__ void __launch_bounds__(256) loss_mean_kernel(const float* __restrict__ loss_n, int N, float* __restrict__ out) {
  __shared__ double sm[256];
  double s = 0.0;
  for (int i = threadIdx.x; i < N; i += 256) s += (double)loss_n[i];
  sm[threadIdx.x] = s;
  __syncthreads();
  for (int w = 128; w > 0; w >>= 1) {
    if (threadIdx.x < w) sm[threadIdx.x] += sm[threadIdx.x + w];
    __syncthreads();
  }
  if (threadIdx.x == 0) out[0] = (float)(sm[0] / (double)N);
}

// dW[j][f] = sum_n dlogits[n][j] * feat[n][f] ; the extra column f == F is the bias gradient
// LBW_TJ: classes per block of the weight gradient (more when that still leaves a few blocks per CU)
template <int LBW_TJ>
__global__ void __launch_bounds__(256) linear_bwd_w_kernel(const float* __restrict__ dlogits, const float* __restrict__ feat,
                                                           float* __restrict__ dw, float* __restrict__ db, int N, int F, int J) {
  // block = LBW_TJ classes and 64 consecutive features (feature index F stands for the bias); the four wavefronts take
  // samples n = wave, wave + 4, ... and their sums are added in a fixed order.  (One class per block read the features
  // once per class.)
  __shared__ float red[LBW_TJ][4][64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int j0 = blockIdx.y * LBW_TJ, f = blockIdx.x * 64 + lane;
  const bool isw = f < F;
  const float* fp = feat + (isw ? f : 0);
  const float one = f == F ? 1.f : 0.f;
  float acc[LBW_TJ];
#pragma unroll
  for (int c = 0; c < LBW_TJ; ++c) acc[c] = 0.f;
  int jc[LBW_TJ];
#pragma unroll
  for (int c = 0; c < LBW_TJ; ++c) jc[c] = j0 + c < J ? j0 + c : j0;
#pragma unroll 8
  for (int n = wave; n < N; n += 4) {
    const float v = isw ? fp[(int64_t)n * F] : one;
    const float* dl = dlogits + (int64_t)n * J;
#pragma unroll
    for (int c = 0; c < LBW_TJ; ++c) acc[c] = __fmaf_rn(dl[jc[c]], v, acc[c]);
  }
#pragma unroll
  for (int c = 0; c < LBW_TJ; ++c) red[c][wave][lane] = acc[c];
  __syncthreads();
  if (wave == 0) {
#pragma unroll
    for (int c = 0; c < LBW_TJ; ++c) {
      if (j0 + c >= J) break;
      const float s = ((red[c][0][lane] + red[c][1][lane]) + red[c][2][lane]) + red[c][3][lane];
      if (isw) dw[(int64_t)(j0 + c) * F + f] = s;
      else if (f == F) db[j0 + c] = s;
    }
  }
}

// dfeat[n][f] = sum_j dlogits[n][j] * w[j][f], classes in ascending order; a thread owns one feature of 8 samples, so a
// weight value is loaded once per eight sums
template <int LBX_TN>
__global__ void __launch_bounds__(256) linear_bwd_x_kernel(const float* __restrict__ dlogits, const float* __restrict__ w,
                                                           float* __restrict__ dfeat, int N, int F, int J) {
  const int f = blockIdx.x * 256 + threadIdx.x;
  const int n0 = blockIdx.y * LBX_TN;
  if (f >= F) return;
  const float* dl[LBX_TN];
#pragma unroll
  for (int s = 0; s < LBX_TN; ++s) dl[s] = dlogits + (int64_t)(n0 + s < N ? n0 + s : n0) * J;
  float acc[LBX_TN];
#pragma unroll
  for (int s = 0; s < LBX_TN; ++s) acc[s] = 0.f;
  for (int j = 0; j < J; ++j) {
    const float v = w[(int64_t)j * F + f];
#pragma unroll
    for (int s = 0; s < LBX_TN; ++s) acc[s] = __fmaf_rn(dl[s][j], v, acc[s]);
  }
#pragma unroll
  for (int s = 0; s < LBX_TN; ++s)
    if (n0 + s < N) dfeat[(int64_t)(n0 + s) * F + f] = acc[s];
}

template <class T>
__global__ void head_feat_bwd_kernel(const float* __restrict__ dfeat, T* __restrict__ dx, int64_t total, int HW, int C, int gap) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= total) return;
  if (!gap) { dx[i] = from_f32<T>(dfeat[i]); return; }
  const int c = (int)(i % C);
  const int64_t n = i / ((int64_t)HW * C);
  dx[i] = from_f32<T>(dfeat[n * C + c] / (float)HW);
}

// GAP backward for channel counts that are a multiple of V: block (chunk of rows, image n); a thread owns V channels,
// reads their gradient once and writes it to every TY-th pixel of the block's rows (16-byte stores, no divisions
// per element)
template <class T, int V>
__global__ void __launch_bounds__(256) gap_bwd_rows_kernel(const float* __restrict__ dfeat, T* __restrict__ dx, int HW, int C,
                                                           int rows_per_block) {
  const int CG = C / V;
  const int TX = CG < 256 ? CG : 256;
  const int TY = 256 / TX;
  const int tx = threadIdx.x % TX, ty = threadIdx.x / TX;
  const int n = blockIdx.y;
  const int p0 = blockIdx.x * rows_per_block;
  const int p1 = p0 + rows_per_block < HW ? p0 + rows_per_block : HW;
  if (ty >= TY) return;
  for (int cg = tx; cg < CG; cg += TX) {
    float v[V];
#pragma unroll
    for (int k = 0; k < V; ++k) v[k] = dfeat[(int64_t)n * C + cg * V + k] / (float)HW;
    Vec<T, V> t;
#pragma unroll
    for (int k = 0; k < V; ++k) t.v[k] = from_f32<T>(v[k]);
    T* base = dx + ((int64_t)n * HW) * C + cg * V;
    for (int p = p0 + ty; p < p1; p += TY) *reinterpret_cast<Vec<T, V>*>(base + (int64_t)p * C) = t;
  }
}

template <class T>
static void launch_feat_bwd(hipStream_t st, const float* dfeat, void* dx, int N, int HW, int C, int gap) {
  constexpr int V = 16 / (int)sizeof(T);
  const int64_t total = (int64_t)N * HW * C;
  if (gap && C % V == 0 && HW >= 64) {
    const int rows_per_block = 64;
    OSEQ_LAUNCH((gap_bwd_rows_kernel<T, V>), dim3(ceil_div(HW, rows_per_block), N), dim3(256), 0, st, dfeat, (T*)dx, HW, C,
                rows_per_block);
  } else {
    OSEQ_LAUNCH(head_feat_bwd_kernel<T>, dim3(ceil_div(total, 256)), dim3(256), 0, st, dfeat, (T*)dx, total, HW, C, gap);
  }
}

void launch_head_logits(hipStream_t st, int dt, const void* x, int N, int HW, int C, int gap, int F, int J, const float* w,
                        const float* b, float* feat, float* logits) {
  const dim3 feat_grid(N, gap ? ceil_div(C, 64) : 1);
  if (dt == DT_F32) OSEQ_LAUNCH(head_feat_kernel<float>, feat_grid, dim3(256), 0, st, (const float*)x, feat, HW, C, gap);
  else if (dt == DT_BF16) OSEQ_LAUNCH(head_feat_kernel<bf16_t>, feat_grid, dim3(256), 0, st, (const bf16_t*)x, feat, HW, C, gap);
  else OSEQ_LAUNCH(head_feat_kernel<f16_t>, feat_grid, dim3(256), 0, st, (const f16_t*)x, feat, HW, C, gap);
  if ((int64_t)ceil_div(N, 8) * ceil_div(J, 8) >= 2048)
    OSEQ_LAUNCH((linear_fwd_kernel<8, 8>), dim3(ceil_div((int64_t)ceil_div(N, 8) * ceil_div(J, 8), 4)), dim3(256), 0, st, feat, w,
                b, logits, N, F, J);
  else
    OSEQ_LAUNCH((linear_fwd_kernel<1, 1>), dim3(ceil_div((int64_t)N * J, 4)), dim3(256), 0, st, feat, w, b, logits, N, F, J);
}

void launch_head_fwd(hipStream_t st, int dt, const void* x, int N, int HW, int C, int gap, int F, int J, const float* w,
                     const float* b, const int32_t* y, float gscale, float* feat, float* logits, float* dlogits,
                     float* loss_n, float* loss_out, int* flags) {
  launch_head_logits(st, dt, x, N, HW, C, gap, F, J, w, b, feat, logits);
  OSEQ_LAUNCH(softmax_ce_kernel, dim3(ceil_div(N, 4)), dim3(256), 0, st, logits, y, loss_n, dlogits, N, J, gscale, flags);
  OSEQ_LAUNCH(loss_mean_kernel, dim3(1), dim3(256), 0, st, loss_n, N, loss_out);
}

void launch_head_bwd(hipStream_t st, int dt, const float* feat, const float* dlogits, const float* w, int N, int HW, int C,
                     int gap, int F, int J, float* dw, float* db, float* dfeat, void* dx) {
  const int strips = ceil_div(F + 1, 64);
  if ((int64_t)strips * ceil_div(J, 4) >= 512)
    OSEQ_LAUNCH(linear_bwd_w_kernel<4>, dim3(strips, ceil_div(J, 4)), dim3(256), 0, st, dlogits, feat, dw, db, N, F, J);
  else
    OSEQ_LAUNCH(linear_bwd_w_kernel<1>, dim3(strips, J), dim3(256), 0, st, dlogits, feat, dw, db, N, F, J);
  if (!dx) return;
  if ((int64_t)ceil_div(F, 256) * ceil_div(N, 8) >= 512)
    OSEQ_LAUNCH(linear_bwd_x_kernel<8>, dim3(ceil_div(F, 256), ceil_div(N, 8)), dim3(256), 0, st, dlogits, w, dfeat, N, F, J);
  else
    OSEQ_LAUNCH(linear_bwd_x_kernel<1>, dim3(ceil_div(F, 256), N), dim3(256), 0, st, dlogits, w, dfeat, N, F, J);
  if (dt == DT_F32) launch_feat_bwd<float>(st, dfeat, dx, N, HW, C, gap);
  else if (dt == DT_BF16) launch_feat_bwd<bf16_t>(st, dfeat, dx, N, HW, C, gap);
  else launch_feat_bwd<f16_t>(st, dfeat, dx, N, HW, C, gap);
}

}  // namespace oseq
