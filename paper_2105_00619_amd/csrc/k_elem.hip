// HBM-bound kernels over NHWC tensors viewed as [rows = N*H*W][C]:
//   input cast, per-channel reductions (BatchNorm statistics, BatchNorm backward sums, bias gradient),
//   BatchNorm apply (+skip, +ReLU), BatchNorm backward apply, ReLU backward, 2x2 max-pool forward/backward.
// Every lane moves 16 bytes per access along the channel axis; per-channel sums are reduced in a fixed
// order (lane-private partials -> LDS -> one partial row per block -> one finishing thread per channel,
// in double), so results do not depend on scheduling.
#include "dev_common.h"
#include "kernels.h"

namespace oseq {

// ------------------------------------------------------------------ cast ----
template <class T>
__global__ void cast_in_kernel(const float* __restrict__ x, T* __restrict__ out, int64_t n) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) out[i] = from_f32<T>(x[i]);
}

template <class T>
__global__ void cast_out_kernel(const T* __restrict__ x, float* __restrict__ out, int64_t n) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) out[i] = to_f32(x[i]);
}

// ----------------------------------------------------- column reductions ----
// RED_BN_BWD: ReLU decisions redone from z (or none); _AOUT: from the sign of the block output; _MASK: from the bits
enum { RED_STATS = 0, RED_BN_BWD = 1, RED_BIAS = 2, RED_BN_BWD_AOUT = 3, RED_BN_BWD_MASK = 4 };

struct RedArgs {
  const void* a;       // STATS: z ; BN_BWD: dA ; BIAS: dz
  const void* z;       // BN_BWD: z
  const void* aout;    // BN_BWD with skip: block output (ReLU mask source); else null
  const uint8_t* mask; // BN_BWD: ReLU decisions as bits, byte (row * C + c) / V holds those of V = 16 / sizeof(T) channels;
                       // takes the place of aout (and of the ReLU flag: the bits are applied as they are)
  const float* stats;  // BN_BWD: [4][C] mean, rstd, scale, shift
  float* partial;      // [nblk][2][C]
  int64_t rows;
  int C, relu, nblk, rows_per_block;
};

template <class T, int V, int MODE>
__global__ void __launch_bounds__(256) colreduce_kernel(RedArgs g) {
  extern __shared__ float smem[];  // [2][TY][TX*V]
  const int CG = g.C / V;
  const int TX = CG < 256 ? CG : 256;
  const int TY = 256 / TX;
  const int tx = threadIdx.x % TX, ty = threadIdx.x / TX;
  const int cg = blockIdx.y * TX + tx;
  const bool active = cg < CG && ty < TY;
  const int c0 = cg * V;
  float s0[V], s1[V];
#pragma unroll
  for (int i = 0; i < V; ++i) s0[i] = s1[i] = 0.f;
  constexpr bool BWD = MODE == RED_BN_BWD || MODE == RED_BN_BWD_AOUT || MODE == RED_BN_BWD_MASK;
  float mean[V], rstd[V], scale[V], shift[V];
  if (BWD && active) {
#pragma unroll
    for (int i = 0; i < V; ++i) {
      mean[i] = g.stats[c0 + i]; rstd[i] = g.stats[g.C + c0 + i];
      if (MODE == RED_BN_BWD) { scale[i] = g.stats[2 * g.C + c0 + i]; shift[i] = g.stats[3 * g.C + c0 + i]; }
    }
  }
  const int64_t r0 = (int64_t)blockIdx.x * g.rows_per_block;
  const int64_t r1 = r0 + g.rows_per_block < g.rows ? r0 + g.rows_per_block : g.rows;
  if (active) {
    const T* a = static_cast<const T*>(g.a);
    const T* z = static_cast<const T*>(g.z);
    const T* ao = MODE == RED_BN_BWD_AOUT ? static_cast<const T*>(g.aout) : nullptr;
    const uint8_t* mk = MODE == RED_BN_BWD_MASK ? g.mask : nullptr;
    // (the row loads below are non-temporal: nothing a reduction reads is read again from the cache it would fill --
    // -2 % on the BatchNorm backward of the bottleneck networks; in the apply kernels, whose output the next kernel
    // reads, the same hint slowed that reader down by as much as it gained)
    // one row's contribution, from values already in registers
    auto accumulate = [&](const float (&va)[V], const float (&vz)[V], const float (&vo)[V], unsigned bits) {
      if (MODE == RED_STATS) {
#pragma unroll
        for (int i = 0; i < V; ++i) { s0[i] += va[i]; s1[i] = __fmaf_rn(va[i], va[i], s1[i]); }
      } else if (MODE == RED_BIAS) {
#pragma unroll
        for (int i = 0; i < V; ++i) s0[i] += va[i];
      } else {
#pragma unroll
        for (int i = 0; i < V; ++i) {
          bool on = true;
          if (MODE == RED_BN_BWD_MASK) on = (bits >> i) & 1u;
          else if (MODE == RED_BN_BWD_AOUT) { if (g.relu) on = vo[i] > 0.f; }
          else if (g.relu) on = bn_affine(vz[i], scale[i], shift[i]) > 0.f;
          const float dy = on ? va[i] : 0.f;
          const float xh = (vz[i] - mean[i]) * rstd[i];
          s0[i] += dy; s1[i] = __fmaf_rn(dy, xh, s1[i]);
        }
      }
    };
    // RT rows per trip while RT remain: their loads are all issued before the first value is used; the rows are still
    // added in the same order.  (Two tensors per row in the BatchNorm-backward modes: two rows per trip measured as
    // well as four or a little better, with fewer registers.)
    constexpr int RT = BWD ? 2 : 4;
    int64_t r = r0 + ty;
    for (; r + (RT - 1) * (int64_t)TY < r1; r += RT * (int64_t)TY) {
      float va[RT][V], vz[RT][V], vo[RT][V];
      unsigned mb[RT];
#pragma unroll
      for (int u = 0; u < RT; ++u) {
        const int64_t off = (r + (int64_t)u * TY) * g.C + c0;
        load_f32_nt<T, V>(a + off, va[u]);
        mb[u] = 0u;
        if (BWD) {
          load_f32_nt<T, V>(z + off, vz[u]);
          if (MODE == RED_BN_BWD_MASK) mb[u] = mk[(r + (int64_t)u * TY) * CG + cg];
          else if (MODE == RED_BN_BWD_AOUT) load_f32<T, V>(ao + off, vo[u]);
        }
      }
#pragma unroll
      for (int u = 0; u < RT; ++u) accumulate(va[u], vz[u], vo[u], mb[u]);
    }
    for (; r < r1; r += TY) {
      const int64_t off = r * g.C + c0;
      float va[V], vz[V], vo[V];
      unsigned mb = 0u;
      load_f32_nt<T, V>(a + off, va);
      if (BWD) {
        load_f32_nt<T, V>(z + off, vz);
        if (MODE == RED_BN_BWD_MASK) mb = mk[r * CG + cg];
        else if (MODE == RED_BN_BWD_AOUT) load_f32<T, V>(ao + off, vo);
      }
      accumulate(va, vz, vo, mb);
    }
  }
  const int W = TX * V;
  if (active) {
#pragma unroll
    for (int i = 0; i < V; ++i) { smem[ty * W + tx * V + i] = s0[i]; smem[(TY + ty) * W + tx * V + i] = s1[i]; }
  }
  __syncthreads();
  if (active && ty == 0) {
#pragma unroll
    for (int i = 0; i < V; ++i) {
      float t0 = 0.f, t1 = 0.f;
      for (int y = 0; y < TY; ++y) { t0 += smem[y * W + tx * V + i]; t1 += smem[(TY + y) * W + tx * V + i]; }
      g.partial[((int64_t)blockIdx.x * 2 + 0) * g.C + c0 + i] = t0;
      g.partial[((int64_t)blockIdx.x * 2 + 1) * g.C + c0 + i] = t1;
    }
  }
}

template <class T, int MODE>
static void launch_colreduce_t(hipStream_t st, const RedArgs& g0) {
  RedArgs g = g0;
  const int vmax = 16 / (int)sizeof(T);
  const int V = (g.C % vmax == 0) ? vmax : 1;
  const int CG = g.C / V;
  const int TX = CG < 256 ? CG : 256;
  const int TY = 256 / TX;
  g.rows_per_block = ceil_div(g.rows, g.nblk);
  dim3 grid(g.nblk, ceil_div(CG, TX));
  const size_t sm = (size_t)2 * TY * TX * V * sizeof(float);
  if (V == vmax) OSEQ_LAUNCH((colreduce_kernel<T, 16 / sizeof(T), MODE>), grid, dim3(256), sm, st, g);
  else OSEQ_LAUNCH((colreduce_kernel<T, 1, MODE>), grid, dim3(256), sm, st, g);
}

template <int MODE>
static void launch_colreduce(hipStream_t st, int dt, const RedArgs& g) {
  if (dt == DT_F32) launch_colreduce_t<float, MODE>(st, g);
  else if (dt == DT_BF16) launch_colreduce_t<bf16_t, MODE>(st, g);
  else launch_colreduce_t<f16_t, MODE>(st, g);
}

// finishing kernels: one wavefront per channel; lane l sums the block partials l, l+64, ... in double, then the
// 64 lane sums are combined by a fixed butterfly, so the result is the same on every run
__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}

__device__ __forceinline__ void partial_sums(const float* __restrict__ partial, int nblk, int C, int c, double& s, double& q) {
  const int lane = threadIdx.x & 63;
  s = 0.0; q = 0.0;
  for (int b = lane; b < nblk; b += 64) {
    s += (double)partial[((int64_t)b * 2) * C + c];
    q += (double)partial[((int64_t)b * 2 + 1) * C + c];
  }
  s = wave_sum(s);
  q = wave_sum(q);
}

// Many row blocks (a convolution over a large batch writes one row of sums per 128 pixels): the rows are first added
// in STAT_FOLD_ROWS fixed ranges, with coalesced reads (thread = channel, four rows in flight per block), so that the
// finishing kernel, which walks a channel's column with one wavefront, has only that many rows left.
constexpr int STAT_FOLD_ROWS = 64;
constexpr int STAT_FOLD_MIN = 512;
__global__ void __launch_bounds__(256) stat_fold_kernel(const float* __restrict__ partial, int nblk, int C, int rows_per_range,
                                                        float* __restrict__ folded) {
  __shared__ double red[2][4][64];
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
  const int c = blockIdx.x * 64 + tx;
  const int b0 = blockIdx.y * rows_per_range;
  const int b1 = b0 + rows_per_range < nblk ? b0 + rows_per_range : nblk;
  double s = 0.0, q = 0.0;
  if (c < C) {
    int b = b0 + ty;
    for (; b + 12 < b1; b += 16) {  // four rows of this thread per trip, loads first
      float vs[4], vq[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        vs[u] = partial[((int64_t)(b + 4 * u) * 2) * C + c];
        vq[u] = partial[((int64_t)(b + 4 * u) * 2 + 1) * C + c];
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) { s += (double)vs[u]; q += (double)vq[u]; }
    }
    for (; b < b1; b += 4) {
      s += (double)partial[((int64_t)b * 2) * C + c];
      q += (double)partial[((int64_t)b * 2 + 1) * C + c];
    }
  }
  red[0][ty][tx] = s; red[1][ty][tx] = q;
  __syncthreads();
  if (ty == 0 && c < C) {
    const double ts = ((red[0][0][tx] + red[0][1][tx]) + red[0][2][tx]) + red[0][3][tx];
    const double tq = ((red[1][0][tx] + red[1][1][tx]) + red[1][2][tx]) + red[1][3][tx];
    folded[((int64_t)blockIdx.y * 2) * C + c] = (float)ts;
    folded[((int64_t)blockIdx.y * 2 + 1) * C + c] = (float)tq;
  }
}

__global__ void __launch_bounds__(256) bn_stats_finalize_kernel(const float* __restrict__ partial, int nblk, int C, double m,
                                                                float eps, float mom, const float* __restrict__ gamma,
                                                                const float* __restrict__ beta, float* __restrict__ stats,
                                                                float* __restrict__ running,
                                                                const int* __restrict__ flags) {
  const int c = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (c >= C) return;
  double s, q;
  partial_sums(partial, nblk, C, c, s, q);
  if ((threadIdx.x & 63) != 0) return;
  const double mean = s / m;
  double var = q / m - mean * mean;
  if (var < 0.0) var = 0.0;
  const double rstd = 1.0 / sqrt(var + (double)eps);
  stats[c] = (float)mean;
  stats[C + c] = (float)rstd;
  stats[2 * C + c] = (float)((double)gamma[c] * rstd);
  stats[3 * C + c] = (float)((double)beta[c] - mean * (double)gamma[c] * rstd);
  if (running && !(flags && flags[1])) {  // a step with an invalid label leaves the running statistics alone
    const double unbiased = m > 1.0 ? var * m / (m - 1.0) : var;
    running[c] = (float)((1.0 - mom) * (double)running[c] + mom * mean);
    running[C + c] = (float)((1.0 - mom) * (double)running[C + c] + mom * unbiased);
  }
}

// inference mode: the same four per-channel constants from the running mean and variance
__global__ void __launch_bounds__(256) bn_eval_stats_kernel(const float* __restrict__ running, const float* __restrict__ gamma,
                                                            const float* __restrict__ beta, float eps, int C,
                                                            float* __restrict__ stats) {
  const int c = blockIdx.x * 256 + threadIdx.x;
  if (c >= C) return;
  const double mean = (double)running[c];
  const double rstd = 1.0 / sqrt((double)running[C + c] + (double)eps);
  stats[c] = (float)mean;
  stats[C + c] = (float)rstd;
  stats[2 * C + c] = (float)((double)gamma[c] * rstd);
  stats[3 * C + c] = (float)((double)beta[c] - mean * (double)gamma[c] * rstd);
}

__global__ void __launch_bounds__(256) bn_bwd_finalize_kernel(const float* __restrict__ partial, int nblk, int C, double m,
                                                              float* __restrict__ dgamma, float* __restrict__ dbeta,
                                                              float* __restrict__ coef) {
  const int c = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (c >= C) return;
  double s, q;
  partial_sums(partial, nblk, C, c, s, q);
  if ((threadIdx.x & 63) != 0) return;
  dbeta[c] = (float)s;
  dgamma[c] = (float)q;
  coef[c] = (float)(s / m);
  coef[C + c] = (float)(q / m);
}

__global__ void __launch_bounds__(256) bias_finalize_kernel(const float* __restrict__ partial, int nblk, int C,
                                                            float* __restrict__ dbias) {
  const int c = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (c >= C) return;
  double s, q;
  partial_sums(partial, nblk, C, c, s, q);
  if ((threadIdx.x & 63) == 0) dbias[c] = (float)s;
}

// ------------------------------------------------------------- BN apply -----
// The backward apply kernel is tiled like the column reductions: a thread owns V consecutive channels, keeps their
// per-channel constants in registers and walks the rows of its block (blockIdx.x) with stride TY, two rows per trip
// with all loads of the trip issued before its first store (loads and stores share one in-order counter).  The
// optional tensors are template parameters, so that each variant is straight-line code (also in the forward kernel).
struct RowArgs {
  int64_t rows;
  int C, relu, rows_per_block;
};

// (the forward apply kernel, with one load and one store stream, measured faster as one group of V channels per
// thread; its per-channel constants are fetched as whole vectors)
// mask (with a skip connection, V = 16 / sizeof(T)): byte i receives the ReLU decisions of group i, bit k = output k > 0
template <class T, int V, bool SKIP>
__global__ void __launch_bounds__(256) bn_apply_kernel(const T* __restrict__ z, const float* __restrict__ stats,
                                                       const T* __restrict__ skip, T* __restrict__ out,
                                                       uint8_t* __restrict__ mask, int64_t groups, int C, int relu) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= groups) return;
  const int CG = C / V;
  const int c0 = (int)(i % CG) * V;
  const int64_t off = i * V;
  float vz[V], vs[V], vo[V], scale[V], shift[V];
  load_f32<T, V>(z + off, vz);
  if (SKIP) load_f32<T, V>(skip + off, vs);
  load_f32<float, V>(stats + 2 * C + c0, scale);
  load_f32<float, V>(stats + 3 * C + c0, shift);
#pragma unroll
  for (int k = 0; k < V; ++k) {
    float y = bn_affine(vz[k], scale[k], shift[k]);
    if (SKIP) y = __fadd_rn(y, vs[k]);
    vo[k] = relu ? fmaxf(y, 0.f) : y;
  }
  store_f32<T, V>(out + off, vo);
  if (SKIP && V > 1 && mask) {
    unsigned bits = 0u;
#pragma unroll
    for (int k = 0; k < V; ++k) bits |= (vo[k] > 0.f ? 1u : 0u) << k;
    mask[i] = (uint8_t)bits;
  }
}

// BatchNorm apply (+ReLU) and the 2x2 max-pool that follows it in one pass over z: a thread owns one pooled position
// of V channels, i.e. the four activations of its window.  The activations are rounded to the storage type before the
// maximum is taken, as the separate pooling kernel finds them in memory, so the result is the same bits.  WRITE_A:
// the activations themselves are also kept (they are when backward needs them).
template <class T, int V, bool WRITE_A>
__global__ void __launch_bounds__(256) bn_apply_pool_kernel(const T* __restrict__ z, const float* __restrict__ stats,
                                                            T* __restrict__ a, T* __restrict__ y, int N, int H, int W, int C,
                                                            int relu) {
  const int CG = C / V, P = H / 2, Q = W / 2;
  const int64_t total = (int64_t)N * P * Q * CG;
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= total) return;
  const int cg = (int)(i % CG);
  int64_t t = i / CG;
  const int q = (int)(t % Q); t /= Q;
  const int pp = (int)(t % P);
  const int n = (int)(t / P);
  const int c0 = cg * V;
  const int64_t base = (((int64_t)n * H + 2 * pp) * W + 2 * q) * C + c0;
  const int64_t offs[4] = {0, (int64_t)C, (int64_t)W * C, (int64_t)W * C + C};
  float vz[4][V], scale[V], shift[V];
#pragma unroll
  for (int u = 0; u < 4; ++u) load_f32<T, V>(z + base + offs[u], vz[u]);
  load_f32<float, V>(stats + 2 * C + c0, scale);
  load_f32<float, V>(stats + 3 * C + c0, shift);
  float m[V];
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    float va[V];
#pragma unroll
    for (int k = 0; k < V; ++k) {
      const float yv = bn_affine(vz[u][k], scale[k], shift[k]);
      va[k] = to_f32(from_f32<T>(relu ? fmaxf(yv, 0.f) : yv));
      m[k] = (u == 0 || va[k] > m[k]) ? va[k] : m[k];
    }
    if (WRITE_A) store_f32<T, V>(a + base + offs[u], va);
  }
  store_f32<T, V>(y + i * V, m);
}

// AOUT: the ReLU mask comes from the block output (a residual sum) instead of being rebuilt from z; DSKIP: the masked
// gradient is also written out for the skip branch
// MS: where the ReLU decisions come from: 0 redone from z, 1 the sign of the block output aout, 2 the bits of mask
template <class T, int V, int MS, bool DSKIP>
__global__ void __launch_bounds__(256) bn_bwd_apply_kernel(const T* __restrict__ da, const T* __restrict__ z,
                                                           const T* __restrict__ aout, const uint8_t* __restrict__ mask,
                                                           const float* __restrict__ stats,
                                                           const float* __restrict__ coef, T* __restrict__ dz,
                                                           T* __restrict__ dskip, RowArgs g) {
  const int CG = g.C / V;
  const int TX = CG < 256 ? CG : 256;
  const int TY = 256 / TX;
  const int tx = threadIdx.x % TX, ty = threadIdx.x / TX;
  const int cg = blockIdx.y * TX + tx;
  if (cg >= CG || ty >= TY) return;
  const int c0 = cg * V;
  constexpr bool AOUT = MS == 1;
  float mean[V], rstd[V], scale[V], shift[V], cb[V], cg2[V];
#pragma unroll
  for (int k = 0; k < V; ++k) {
    const int c = c0 + k;
    mean[k] = stats[c]; rstd[k] = stats[g.C + c]; scale[k] = stats[2 * g.C + c]; shift[k] = stats[3 * g.C + c];
    cb[k] = coef[c]; cg2[k] = coef[g.C + c];
  }
  const int64_t r0 = (int64_t)blockIdx.x * g.rows_per_block;
  const int64_t r1 = r0 + g.rows_per_block < g.rows ? r0 + g.rows_per_block : g.rows;
  auto one = [&](const float (&va)[V], const float (&vz)[V], const float (&vo)[V], unsigned bits, float (&rz)[V],
                 float (&rs)[V]) {
#pragma unroll
    for (int k = 0; k < V; ++k) {
      bool on = true;
      if (MS == 2) on = (bits >> k) & 1u;
      else if (g.relu) on = AOUT ? (vo[k] > 0.f) : (bn_affine(vz[k], scale[k], shift[k]) > 0.f);
      const float dy = on ? va[k] : 0.f;
      const float xh = (vz[k] - mean[k]) * rstd[k];
      rz[k] = scale[k] * (dy - cb[k] - xh * cg2[k]);
      rs[k] = dy;
    }
  };
  // two rows per trip, all loads before the stores (four rows: 575 against 544 us for the whole backward of a block
  // output at 262 144 x 1024, bf16; one row: 550)
  constexpr int RT = 2;
  int64_t r = r0 + ty;
  for (; r + (RT - 1) * (int64_t)TY < r1; r += RT * (int64_t)TY) {
    float va[RT][V], vz[RT][V], vo[RT][V], rz[RT][V], rs[RT][V];
    unsigned mb[RT];
#pragma unroll
    for (int u = 0; u < RT; ++u) {
      const int64_t off = (r + (int64_t)u * TY) * g.C + c0;
      load_f32<T, V>(da + off, va[u]);
      load_f32<T, V>(z + off, vz[u]);
      if (AOUT) load_f32<T, V>(aout + off, vo[u]);
      mb[u] = MS == 2 ? mask[(r + (int64_t)u * TY) * CG + cg] : 0u;
    }
#pragma unroll
    for (int u = 0; u < RT; ++u) one(va[u], vz[u], vo[u], mb[u], rz[u], rs[u]);
#pragma unroll
    for (int u = 0; u < RT; ++u) {
      const int64_t off = (r + (int64_t)u * TY) * g.C + c0;
      store_f32<T, V>(dz + off, rz[u]);
      if (DSKIP) store_f32<T, V>(dskip + off, rs[u]);
    }
  }
  for (; r < r1; r += TY) {
    const int64_t off = r * g.C + c0;
    float va[V], vz[V], vo[V], rz[V], rs[V];
    unsigned mb = 0u;
    load_f32<T, V>(da + off, va);
    load_f32<T, V>(z + off, vz);
    if (AOUT) load_f32<T, V>(aout + off, vo);
    if (MS == 2) mb = mask[r * CG + cg];
    one(va, vz, vo, mb, rz, rs);
    store_f32<T, V>(dz + off, rz);
    if (DSKIP) store_f32<T, V>(dskip + off, rs);
  }
}

// ---- BatchNorm(+ReLU) backward through the 2x2 max-pool behind it ---------------------------------------------
// The pool's backward, the gradient it would write (dA, full resolution) and the activation it would read are all
// skipped: a thread owns one pooled position of V channels, reads the four z of its window and the pooled gradient,
// rebuilds the four activations as the forward kernel computed them (rounded to the storage type), finds the first
// maximum in scan order, and so knows dA at its four positions.  Two kernels with the same tiling: the per-channel
// sums (as colreduce: row blocks of pooled positions, partial [nblk][2][C]) and, after the finishing kernel, dz.
struct PoolBwdArgs {
  int64_t rows;  // pooled positions N * P * Q
  int C, relu, rows_per_block, W, Q, PQ, HW;  // full-resolution width, pooled width, pooled / full positions per image
};

template <class T, int V>
__device__ __forceinline__ void pool_window_grad(const T* __restrict__ z, const T* __restrict__ dy, int64_t r, int c0,
                                                 const PoolBwdArgs& g, const float (&scale)[V], const float (&shift)[V],
                                                 float (&vz)[4][V], float (&dyv)[4][V], int64_t (&off)[4]) {
  const int64_t n = r / g.PQ;
  const int rem = (int)(r - n * g.PQ);
  const int p = rem / g.Q, q = rem - p * g.Q;
  off[0] = ((n * g.HW + (int64_t)(2 * p) * g.W + 2 * q)) * g.C + c0;
  off[1] = off[0] + g.C; off[2] = off[0] + (int64_t)g.W * g.C; off[3] = off[2] + g.C;
  float gy[V];
#pragma unroll
  for (int u = 0; u < 4; ++u) load_f32<T, V>(z + off[u], vz[u]);
  load_f32<T, V>(dy + r * g.C + c0, gy);
#pragma unroll
  for (int k = 0; k < V; ++k) {
    float y[4], m = 0.f;
    int arg = 0;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      y[u] = bn_affine(vz[u][k], scale[k], shift[k]);
      const float a = to_f32(from_f32<T>(g.relu ? fmaxf(y[u], 0.f) : y[u]));
      if (u == 0 || a > m) { m = a; arg = u; }
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const bool on = !g.relu || y[u] > 0.f;
      dyv[u][k] = (arg == u && on) ? gy[k] : 0.f;
    }
  }
}

template <class T, int V>
__global__ void __launch_bounds__(256) bn_bwd_pool_reduce_kernel(const T* __restrict__ dy, const T* __restrict__ z,
                                                                 const float* __restrict__ stats, float* __restrict__ partial,
                                                                 PoolBwdArgs g) {
  extern __shared__ float smem[];  // [2][TY][TX*V]
  const int CG = g.C / V;
  const int TX = CG < 256 ? CG : 256;
  const int TY = 256 / TX;
  const int tx = threadIdx.x % TX, ty = threadIdx.x / TX;
  const int cg = blockIdx.y * TX + tx;
  const bool active = cg < CG && ty < TY;
  const int c0 = cg * V;
  float s0[V], s1[V];
#pragma unroll
  for (int i = 0; i < V; ++i) s0[i] = s1[i] = 0.f;
  if (active) {
    float mean[V], rstd[V], scale[V], shift[V];
#pragma unroll
    for (int i = 0; i < V; ++i) {
      mean[i] = stats[c0 + i]; rstd[i] = stats[g.C + c0 + i];
      scale[i] = stats[2 * g.C + c0 + i]; shift[i] = stats[3 * g.C + c0 + i];
    }
    const int64_t r0 = (int64_t)blockIdx.x * g.rows_per_block;
    const int64_t r1 = r0 + g.rows_per_block < g.rows ? r0 + g.rows_per_block : g.rows;
    for (int64_t r = r0 + ty; r < r1; r += TY) {
      float vz[4][V], dyv[4][V];
      int64_t off[4];
      pool_window_grad<T, V>(z, dy, r, c0, g, scale, shift, vz, dyv, off);
#pragma unroll
      for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int i = 0; i < V; ++i) {
          const float xh = (vz[u][i] - mean[i]) * rstd[i];
          s0[i] += dyv[u][i]; s1[i] = __fmaf_rn(dyv[u][i], xh, s1[i]);
        }
    }
  }
  const int W = TX * V;
  if (active) {
#pragma unroll
    for (int i = 0; i < V; ++i) { smem[ty * W + tx * V + i] = s0[i]; smem[(TY + ty) * W + tx * V + i] = s1[i]; }
  }
  __syncthreads();
  if (active && ty == 0) {
#pragma unroll
    for (int i = 0; i < V; ++i) {
      float t0 = 0.f, t1 = 0.f;
      for (int y = 0; y < TY; ++y) { t0 += smem[y * W + tx * V + i]; t1 += smem[(TY + y) * W + tx * V + i]; }
      partial[((int64_t)blockIdx.x * 2 + 0) * g.C + c0 + i] = t0;
      partial[((int64_t)blockIdx.x * 2 + 1) * g.C + c0 + i] = t1;
    }
  }
}

template <class T, int V>
__global__ void __launch_bounds__(256) bn_bwd_pool_apply_kernel(const T* __restrict__ dy, const T* __restrict__ z,
                                                                const float* __restrict__ stats, const float* __restrict__ coef,
                                                                T* __restrict__ dz, PoolBwdArgs g) {
  const int CG = g.C / V;
  const int TX = CG < 256 ? CG : 256;
  const int TY = 256 / TX;
  const int tx = threadIdx.x % TX, ty = threadIdx.x / TX;
  const int cg = blockIdx.y * TX + tx;
  if (cg >= CG || ty >= TY) return;
  const int c0 = cg * V;
  float mean[V], rstd[V], scale[V], shift[V], cb[V], cg2[V];
#pragma unroll
  for (int k = 0; k < V; ++k) {
    const int c = c0 + k;
    mean[k] = stats[c]; rstd[k] = stats[g.C + c]; scale[k] = stats[2 * g.C + c]; shift[k] = stats[3 * g.C + c];
    cb[k] = coef[c]; cg2[k] = coef[g.C + c];
  }
  const int64_t r0 = (int64_t)blockIdx.x * g.rows_per_block;
  const int64_t r1 = r0 + g.rows_per_block < g.rows ? r0 + g.rows_per_block : g.rows;
  for (int64_t r = r0 + ty; r < r1; r += TY) {
    float vz[4][V], dyv[4][V];
    int64_t off[4];
    pool_window_grad<T, V>(z, dy, r, c0, g, scale, shift, vz, dyv, off);
    float rz[4][V];
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
      for (int k = 0; k < V; ++k) {
        const float xh = (vz[u][k] - mean[k]) * rstd[k];
        rz[u][k] = scale[k] * (dyv[u][k] - cb[k] - xh * cg2[k]);
      }
#pragma unroll
    for (int u = 0; u < 4; ++u) store_f32<T, V>(dz + off[u], rz[u]);
  }
}

template <class T, int V>
__global__ void __launch_bounds__(256) relu_bwd_kernel(const T* __restrict__ da, const T* __restrict__ a,
                                                       T* __restrict__ dz, int64_t groups) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= groups) return;
  float va[V], vo[V], r[V];
  load_f32<T, V>(da + i * V, va);
  load_f32<T, V>(a + i * V, vo);
#pragma unroll
  for (int k = 0; k < V; ++k) r[k] = vo[k] > 0.f ? va[k] : 0.f;
  store_f32<T, V>(dz + i * V, r);
}

// -------------------------------------------------------------- max-pool ----
template <class T, int V>
__global__ void __launch_bounds__(256) maxpool_fwd_kernel(const T* __restrict__ x, T* __restrict__ y, int N, int H, int W,
                                                          int C, int P, int Q) {
  const int CG = C / V;
  const int64_t total = (int64_t)N * P * Q * CG;
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= total) return;
  const int cg = (int)(i % CG);
  int64_t t = i / CG;
  const int q = (int)(t % Q); t /= Q;
  const int p = (int)(t % P);
  const int n = (int)(t / P);
  const T* base = x + (((int64_t)n * H + 2 * p) * W + 2 * q) * C + cg * V;
  float m[V], v[V];
  load_f32<T, V>(base, m);
  load_f32<T, V>(base + C, v);
#pragma unroll
  for (int k = 0; k < V; ++k) m[k] = v[k] > m[k] ? v[k] : m[k];
  load_f32<T, V>(base + (int64_t)W * C, v);
#pragma unroll
  for (int k = 0; k < V; ++k) m[k] = v[k] > m[k] ? v[k] : m[k];
  load_f32<T, V>(base + (int64_t)W * C + C, v);
#pragma unroll
  for (int k = 0; k < V; ++k) m[k] = v[k] > m[k] ? v[k] : m[k];
  store_f32<T, V>(y + i * V, m);
}

// One thread per input position: the gradient of its window goes to the first maximum in scan order.
template <class T, int V>
__global__ void __launch_bounds__(256) maxpool_bwd_kernel(const T* __restrict__ x, const T* __restrict__ dy,
                                                          T* __restrict__ dx, int N, int H, int W, int C, int P, int Q) {
  const int CG = C / V;
  const int64_t total = (int64_t)N * H * W * CG;
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= total) return;
  const int cg = (int)(i % CG);
  int64_t t = i / CG;
  const int w = (int)(t % W); t /= W;
  const int h = (int)(t % H);
  const int n = (int)(t / H);
  float r[V];
#pragma unroll
  for (int k = 0; k < V; ++k) r[k] = 0.f;
  const int p = h >> 1, q = w >> 1;
  if (p < P && q < Q) {
    const T* base = x + (((int64_t)n * H + 2 * p) * W + 2 * q) * C + cg * V;
    float m[V], v[V], g[V];
    int arg[V];
    load_f32<T, V>(base, m);
#pragma unroll
    for (int k = 0; k < V; ++k) arg[k] = 0;
    load_f32<T, V>(base + C, v);
#pragma unroll
    for (int k = 0; k < V; ++k) if (v[k] > m[k]) { m[k] = v[k]; arg[k] = 1; }
    load_f32<T, V>(base + (int64_t)W * C, v);
#pragma unroll
    for (int k = 0; k < V; ++k) if (v[k] > m[k]) { m[k] = v[k]; arg[k] = 2; }
    load_f32<T, V>(base + (int64_t)W * C + C, v);
#pragma unroll
    for (int k = 0; k < V; ++k) if (v[k] > m[k]) { m[k] = v[k]; arg[k] = 3; }
    load_f32<T, V>(dy + (((int64_t)n * P + p) * Q + q) * C + cg * V, g);
    const int me = (h & 1) * 2 + (w & 1);
#pragma unroll
    for (int k = 0; k < V; ++k) r[k] = arg[k] == me ? g[k] : 0.f;
  }
  store_f32<T, V>(dx + i * V, r);
}

// ---------------------------------------------------------------- launch ----
#define DISPATCH_TV(dt, C, CALL)                                               \
  do {                                                                         \
    if (dt == DT_F32) { if ((C) % 4 == 0) { CALL(float, 4); } else { CALL(float, 1); } } \
    else if (dt == DT_BF16) { if ((C) % 8 == 0) { CALL(bf16_t, 8); } else { CALL(bf16_t, 1); } } \
    else { if ((C) % 8 == 0) { CALL(f16_t, 8); } else { CALL(f16_t, 1); } }     \
  } while (0)

void launch_cast_in(hipStream_t st, int dt, const float* x, void* out, int64_t n) {
  const int blocks = (int)((n + 255) / 256 < 4096 ? (n + 255) / 256 : 4096);
  if (dt == DT_F32) OSEQ_LAUNCH(cast_in_kernel<float>, dim3(blocks), dim3(256), 0, st, x, (float*)out, n);
  else if (dt == DT_BF16) OSEQ_LAUNCH(cast_in_kernel<bf16_t>, dim3(blocks), dim3(256), 0, st, x, (bf16_t*)out, n);
  else OSEQ_LAUNCH(cast_in_kernel<f16_t>, dim3(blocks), dim3(256), 0, st, x, (f16_t*)out, n);
}

void launch_cast_out(hipStream_t st, int dt, const void* x, float* out, int64_t n) {
  const int blocks = (int)((n + 255) / 256 < 4096 ? (n + 255) / 256 : 4096);
  if (dt == DT_F32) OSEQ_LAUNCH(cast_out_kernel<float>, dim3(blocks), dim3(256), 0, st, (const float*)x, out, n);
  else if (dt == DT_BF16) OSEQ_LAUNCH(cast_out_kernel<bf16_t>, dim3(blocks), dim3(256), 0, st, (const bf16_t*)x, out, n);
  else OSEQ_LAUNCH(cast_out_kernel<f16_t>, dim3(blocks), dim3(256), 0, st, (const f16_t*)x, out, n);
}

void launch_bn_stats(hipStream_t st, int dt, const void* z, int64_t rows, int C, int nblk, float* partial, float eps,
                     float mom, const float* gamma, const float* beta, float* stats, float* running,
                     const int* flags) {
  RedArgs g{}; g.a = z; g.partial = partial; g.rows = rows; g.C = C; g.nblk = nblk;
  launch_colreduce<RED_STATS>(st, dt, g);
  OSEQ_LAUNCH(bn_stats_finalize_kernel, dim3(ceil_div(C, 4)), dim3(256), 0, st, partial, nblk, C, (double)rows,
                     eps, mom, gamma, beta, stats, running, flags);
}

int bn_stats_fold_rows(int nblk) { return nblk >= STAT_FOLD_MIN ? STAT_FOLD_ROWS : 0; }

// partial: [nblk][2][C] block sums, followed by room for [bn_stats_fold_rows(nblk)][2][C] floats
void launch_bn_stats_finalize(hipStream_t st, float* partial, int64_t rows, int C, int nblk, float eps, float mom,
                              const float* gamma, const float* beta, float* stats, float* running,
                              const int* flags) {
  if (bn_stats_fold_rows(nblk) > 0) {
    float* folded = partial + (int64_t)nblk * 2 * C;
    const int per = ceil_div(nblk, STAT_FOLD_ROWS);
    const int ranges = ceil_div(nblk, per);  // no empty range
    OSEQ_LAUNCH(stat_fold_kernel, dim3(ceil_div(C, 64), ranges), dim3(256), 0, st, partial, nblk, C, per, folded);
    partial = folded;
    nblk = ranges;
  }
  OSEQ_LAUNCH(bn_stats_finalize_kernel, dim3(ceil_div(C, 4)), dim3(256), 0, st, partial, nblk, C, (double)rows,
                     eps, mom, gamma, beta, stats, running, flags);
}

// Row blocks of the apply kernels: eight rows per thread (the per-channel constants are fetched once per block; with
// two-row trips the whole backward of a block output at 262 144 x 1024, bf16, takes 556 / 543 / 532 / 545 / 575 us at
// 32 / 16 / 8 / 4 / 2 rows) when that still leaves about four blocks per CU, else fewer (small tensors), from the
// shape only.
static void row_tiling(int64_t rows, int C, int V, RowArgs& g, dim3& grid) {
  const int CG = C / V;
  const int TX = CG < 256 ? CG : 256;
  const int TY = 256 / TX;
  const int ytiles = ceil_div(CG, TX);
  int per_thread = 8;
  while (per_thread > 1 && (int64_t)ceil_div(rows, (int64_t)TY * per_thread) * ytiles < 1024) per_thread /= 2;
  g.rows = rows; g.C = C; g.rows_per_block = TY * per_thread;
  grid = dim3(ceil_div(rows, g.rows_per_block), ytiles);
}

void launch_bn_eval_stats(hipStream_t st, const float* running, const float* gamma, const float* beta, float eps, int C,
                          float* stats) {
  OSEQ_LAUNCH(bn_eval_stats_kernel, dim3(ceil_div(C, 256)), dim3(256), 0, st, running, gamma, beta, eps, C, stats);
}

void launch_bn_apply(hipStream_t st, int dt, const void* z, const float* stats, const void* skip, void* out, void* mask,
                     int64_t rows, int C, int relu) {
#define CALL(T, V)                                                                                                    \
  { const int64_t groups = rows * (C / V);                                                                             \
    uint8_t* mk = V > 1 ? (uint8_t*)mask : nullptr;                                                                    \
    if (skip) OSEQ_LAUNCH((bn_apply_kernel<T, V, true>), dim3(ceil_div(groups, 256)), dim3(256), 0, st,         \
                                 (const T*)z, stats, (const T*)skip, (T*)out, mk, groups, C, relu);                    \
    else OSEQ_LAUNCH((bn_apply_kernel<T, V, false>), dim3(ceil_div(groups, 256)), dim3(256), 0, st,             \
                            (const T*)z, stats, (const T*)skip, (T*)out, mk, groups, C, relu); }
  DISPATCH_TV(dt, C, CALL);
#undef CALL
}

void launch_bn_apply_pool(hipStream_t st, int dt, const void* z, const float* stats, void* a, void* y, int N, int H, int W,
                          int C, int relu) {
#define CALL(T, V)                                                                                                     \
  { const int64_t total = (int64_t)N * (H / 2) * (W / 2) * (C / V);                                                     \
    if (a) OSEQ_LAUNCH((bn_apply_pool_kernel<T, V, true>), dim3(ceil_div(total, 256)), dim3(256), 0, st, (const T*)z,   \
                       stats, (T*)a, (T*)y, N, H, W, C, relu);                                                          \
    else OSEQ_LAUNCH((bn_apply_pool_kernel<T, V, false>), dim3(ceil_div(total, 256)), dim3(256), 0, st, (const T*)z,    \
                     stats, (T*)a, (T*)y, N, H, W, C, relu); }
  DISPATCH_TV(dt, C, CALL);
#undef CALL
}

void launch_bn_bwd(hipStream_t st, int dt, const void* da, const void* z, const void* aout, const void* mask,
                   const float* stats, int64_t rows, int C, int relu, int nblk, float* ws, float* dgamma, float* dbeta,
                   void* dz, void* dskip) {
  RedArgs g{}; g.a = da; g.z = z; g.aout = aout; g.mask = (const uint8_t*)mask; g.stats = stats; g.partial = ws; g.rows = rows;
  g.C = C; g.relu = relu; g.nblk = nblk;
  // the same choice of the ReLU decisions' source as the apply kernel below makes
  const int vmax = dt == DT_F32 ? 4 : 8;
  if (mask && C % vmax == 0) launch_colreduce<RED_BN_BWD_MASK>(st, dt, g);
  else if (aout) launch_colreduce<RED_BN_BWD_AOUT>(st, dt, g);
  else launch_colreduce<RED_BN_BWD>(st, dt, g);
  float* coef = ws + (int64_t)nblk * 2 * C;
  OSEQ_LAUNCH(bn_bwd_finalize_kernel, dim3(ceil_div(C, 4)), dim3(256), 0, st, ws, nblk, C, (double)rows, dgamma,
                     dbeta, coef);
#define APPLY(T, V, MS, DS)                                                                                             \
  OSEQ_LAUNCH((bn_bwd_apply_kernel<T, V, MS, DS>), grid, dim3(256), 0, st, (const T*)da, (const T*)z,             \
                     (const T*)aout, (const uint8_t*)mask, stats, coef, (T*)dz, (T*)dskip, ra)
#define CALL(T, V)                                                                                                      \
  { RowArgs ra{}; dim3 grid; row_tiling(rows, C, V, ra, grid); ra.relu = relu;                                           \
    if (mask && V > 1) { if (dskip) APPLY(T, V, 2, true); else APPLY(T, V, 2, false); }                                  \
    else if (aout) { if (dskip) APPLY(T, V, 1, true); else APPLY(T, V, 1, false); }                                      \
    else { if (dskip) APPLY(T, V, 0, true); else APPLY(T, V, 0, false); } }
  DISPATCH_TV(dt, C, CALL);
#undef CALL
#undef APPLY
}

// BatchNorm(+ReLU) backward where dy is the gradient of the 2x2 max-pool behind the activation: z [N][H][W][C] (H, W
// even), dy [N][H/2][W/2][C]; ws as for launch_bn_bwd
void launch_bn_bwd_pool(hipStream_t st, int dt, const void* dy, const void* z, const float* stats, int N, int H, int W, int C,
                        int relu, int nblk, float* ws, float* dgamma, float* dbeta, void* dz) {
  PoolBwdArgs g{};
  g.rows = (int64_t)N * (H / 2) * (W / 2); g.C = C; g.relu = relu; g.W = W; g.Q = W / 2; g.PQ = (H / 2) * (W / 2); g.HW = H * W;
  float* coef = ws + (int64_t)nblk * 2 * C;
#define CALL(T, V)                                                                                                       \
  { const int CG = C / V, TX = CG < 256 ? CG : 256, TY = 256 / TX, ytiles = ceil_div(CG, TX);                              \
    PoolBwdArgs gr = g; gr.rows_per_block = ceil_div(g.rows, nblk);                                                        \
    OSEQ_LAUNCH((bn_bwd_pool_reduce_kernel<T, V>), dim3(nblk, ytiles), dim3(256), (size_t)2 * TY * TX * V * sizeof(float), \
                st, (const T*)dy, (const T*)z, stats, ws, gr);                                                             \
    OSEQ_LAUNCH(bn_bwd_finalize_kernel, dim3(ceil_div(C, 4)), dim3(256), 0, st, ws, nblk, C, (double)N * H * W, dgamma,    \
                dbeta, coef);                                                                                              \
    PoolBwdArgs ga = g; int per = 2;                                                                                       \
    while (per > 1 && (int64_t)ceil_div(g.rows, (int64_t)TY * per) * ytiles < 1024) per /= 2;                              \
    ga.rows_per_block = TY * per;                                                                                          \
    OSEQ_LAUNCH((bn_bwd_pool_apply_kernel<T, V>), dim3(ceil_div(g.rows, ga.rows_per_block), ytiles), dim3(256), 0, st,     \
                (const T*)dy, (const T*)z, stats, coef, (T*)dz, ga); }
  DISPATCH_TV(dt, C, CALL);
#undef CALL
}

void launch_relu_bwd(hipStream_t st, int dt, const void* da, const void* a, void* dz, int64_t rows, int C) {
#define CALL(T, V)                                                                                                  \
  { const int64_t groups = rows * (C / V);                                                                           \
    OSEQ_LAUNCH((relu_bwd_kernel<T, V>), dim3(ceil_div(groups, 256)), dim3(256), 0, st, (const T*)da,         \
                       (const T*)a, (T*)dz, groups); }
  DISPATCH_TV(dt, C, CALL);
#undef CALL
}

void launch_bias_grad(hipStream_t st, int dt, const void* dz, int64_t rows, int C, int nblk, float* partial, float* dbias) {
  RedArgs g{}; g.a = dz; g.partial = partial; g.rows = rows; g.C = C; g.nblk = nblk;
  launch_colreduce<RED_BIAS>(st, dt, g);
  OSEQ_LAUNCH(bias_finalize_kernel, dim3(ceil_div(C, 4)), dim3(256), 0, st, partial, nblk, C, dbias);
}

void launch_maxpool_fwd(hipStream_t st, int dt, const void* x, void* y, int N, int H, int W, int C) {
  const int P = H / 2, Q = W / 2;
#define CALL(T, V)                                                                                                  \
  { const int64_t total = (int64_t)N * P * Q * (C / V);                                                              \
    OSEQ_LAUNCH((maxpool_fwd_kernel<T, V>), dim3(ceil_div(total, 256)), dim3(256), 0, st, (const T*)x, (T*)y, \
                       N, H, W, C, P, Q); }
  DISPATCH_TV(dt, C, CALL);
#undef CALL
}

void launch_maxpool_bwd(hipStream_t st, int dt, const void* x, const void* dy, void* dx, int N, int H, int W, int C) {
  const int P = H / 2, Q = W / 2;
#define CALL(T, V)                                                                                                  \
  { const int64_t total = (int64_t)N * H * W * (C / V);                                                              \
    OSEQ_LAUNCH((maxpool_bwd_kernel<T, V>), dim3(ceil_div(total, 256)), dim3(256), 0, st, (const T*)x,        \
                       (const T*)dy, (T*)dx, N, H, W, C, P, Q); }
  DISPATCH_TV(dt, C, CALL);
#undef CALL
}

}  // namespace oseq
