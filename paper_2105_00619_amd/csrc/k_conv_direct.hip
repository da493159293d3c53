// Direct (plain FMA) convolution forward / data gradient / weight gradient for shapes the matrix-core
// kernels do not take: very few channels (the 3-channel stem, the tiny test networks).  NHWC activations,
// (C_out, kh, kw, C_in) weights, fp32 accumulation in a fixed order.
#include "dev_common.h"
#include "epilogue.h"
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
                                                              ConvGeom g, int relu, FastDiv divQ, FastDiv divPQ) {
  // block = 128 pixels x 64 output channels (blockIdx.y selects the group of 64); thread = 4 pixels x 8 channels,
  // the 8 threads of a pixel next to each other so that a wavefront writes 8 whole rows of 64 channels, and every
  // weight read from LDS serves four pixels.  The 8 threads of a pixel share the loading of its R*S*C inputs
  // through LDS (vector-memory instructions, not bytes, bound this kernel otherwise).
  constexpr int RSC = 9 * C;  // 3x3 filter
  constexpr int XP = (RSC + 3) / 4 * 4;
  constexpr int PPT = 4;
  __shared__ __attribute__((aligned(16))) float ws[RSC * 64];        // [e][channel]
  __shared__ __attribute__((aligned(16))) float xs[32 * PPT * XP];   // [pixel of the block][e]
  const int kbase = blockIdx.y * 64;
  const int kn = g.K - kbase < 64 ? g.K - kbase : 64;
  for (int i = threadIdx.x; i < RSC * 64; i += 256) {
    const int k = i / RSC, e = i - k * RSC;  // consecutive threads read consecutive weights
    ws[e * 64 + k] = k < kn ? to_f32(w[(kbase + k) * RSC + e]) : 0.f;
  }
  const int grp = threadIdx.x & 7, slot = threadIdx.x >> 3;
  const int pixels = g.N * g.P * g.Q;  // < 2^24 (checked by the launcher), so 32-bit index arithmetic throughout
  const int H = g.H, W = g.W, cstride = g.stride, pad = g.pad;
  int m[PPT];
  // this thread's input elements e = grp + 8u of each of its pixels: filter offsets and channel are pixel-independent
  int er[(RSC + 7) / 8], es[(RSC + 7) / 8], ec[(RSC + 7) / 8];
#pragma unroll
  for (int u = 0; u < (RSC + 7) / 8; ++u) {
    const int e = grp + 8 * u < RSC ? grp + 8 * u : RSC - 1;
    const int tap = e / C;
    ec[u] = e - tap * C; er[u] = tap / 3 - pad; es[u] = tap % 3 - pad;
  }
#pragma unroll
  for (int i = 0; i < PPT; ++i) {
    m[i] = blockIdx.x * (32 * PPT) + slot + 32 * i;
    const uint32_t mm = m[i] < pixels ? (uint32_t)m[i] : 0u;
    const uint32_t n = divPQ.div(mm), rem = mm - n * divPQ.d;
    const uint32_t p = divQ.div(rem), q = rem - p * divQ.d;
    const int ih0 = (int)p * cstride, iw0 = (int)q * cstride, nbase = (int)n * H;
#pragma unroll
    for (int u = 0; u < (RSC + 7) / 8; ++u) {
      const int ih = ih0 + er[u], iw = iw0 + es[u];
      const bool ok = ih >= 0 && ih < H && iw >= 0 && iw < W;
      const float v = to_f32(x[ok ? ((nbase + ih) * W + iw) * C + ec[u] : 0]);
      if (grp + 8 * u < RSC) xs[(slot + 32 * i) * XP + grp + 8 * u] = ok ? v : 0.f;
    }
  }
  __syncthreads();
  float acc[PPT][8];
#pragma unroll
  for (int i = 0; i < PPT; ++i)
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[i][j] = 0.f;
  // one filter tap (C inputs) per iteration; not unrolled further: with all R*S*C steps visible the compiler
  // hoists every LDS read to the top and parks the values in accumulation registers
#pragma unroll 1
  for (int tap = 0; tap < 9; ++tap) {
#pragma unroll
    for (int c = 0; c < C; ++c) {
      const int e = tap * C + c;
      const float* wp = &ws[e * 64 + grp * 8];
      float wv[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) wv[j] = wp[j];
#pragma unroll
      for (int i = 0; i < PPT; ++i) {
        const float xv = xs[(slot + 32 * i) * XP + e];
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[i][j] = __fmaf_rn(xv, wv[j], acc[i][j]);
      }
    }
  }
  if (grp * 8 >= kn) return;
#pragma unroll
  for (int i = 0; i < PPT; ++i) {
    if (m[i] >= pixels) continue;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      float a = acc[i][j];
      if (bias) a += bias[kbase + grp * 8 + j];
      acc[i][j] = relu ? fmaxf(a, 0.f) : a;
    }
    store_f32<T, 8>(out + (int64_t)m[i] * g.K + kbase + grp * 8, acc[i]);
  }
}

// The same layer in the 16-bit modes, with at most 32 products per output (3x3 on up to 3 channels) and output
// channels in groups of 64: the plain-FMA kernel above is bound by its 27 x 64 multiply-adds per pixel on the vector
// units (296 us for 4.2 M pixels, where writing the output takes 100), so the products go to the matrix cores as one
// 32-deep MFMA step: the block gathers the patches of its 128 pixels into LDS as [pixel][32] in the storage type (depth
// 27..31 zero), the 64 x 32 weight tile beside them, every wavefront multiplies 64 pixels x 32 channels with two
// 32x32x16 MFMAs per 32 x 32 tile, and the shared epilogue rounds and stores whole rows.
template <class T> struct StemMma;
template <> struct StemMma<bf16_t> {
  typedef __attribute__((ext_vector_type(8))) __bf16 V;
  typedef __attribute__((ext_vector_type(16))) float A;
  __device__ static __forceinline__ A run(V a, V b, A c) { return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0); }
};
template <> struct StemMma<f16_t> {
  typedef __attribute__((ext_vector_type(8))) _Float16 V;
  typedef __attribute__((ext_vector_type(16))) float A;
  __device__ static __forceinline__ A run(V a, V b, A c) { return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0); }
};

template <class T, int C>
__global__ void __launch_bounds__(256) conv_fwd_smallc_mfma_kernel(const T* __restrict__ x, const T* __restrict__ w,
                                                                   const float* __restrict__ bias, T* __restrict__ out,
                                                                   ConvGeom g, int relu, FastDiv divQ, FastDiv divPQ) {
  typedef typename StemMma<T>::V FV;
  typedef typename StemMma<T>::A v16f;
  constexpr int RSC = 9 * C;       // <= 32
  constexpr int PITCH = 40;        // elements per LDS row (80 bytes)
  constexpr int PPT = 4;
  static_assert(RSC <= 32, "one 32-deep step");
  // 15 KB of operands, reused as the 17 KB epilogue tile: eight blocks (all 32 wavefronts) fit a CU, which is what hides
  // the latency of the gather (a block is a dozen dependent-free 2-byte loads per thread, a barrier and a few MFMAs)
  constexpr int EP_BYTES = 64 * (64 + 4) * 4, OP_BYTES = (64 + 128) * PITCH * (int)sizeof(T);
  __shared__ __attribute__((aligned(16))) unsigned char smem[EP_BYTES > OP_BYTES ? EP_BYTES : OP_BYTES];
  T* ws = reinterpret_cast<T*>(smem);                 // [channel][depth]
  T* xs = ws + 64 * PITCH;                            // [pixel of the block][depth]
  float* ep = reinterpret_cast<float*>(smem);         // epilogue tile (after the operands have been read)
  const int tid = threadIdx.x;
  const int kbase = blockIdx.y * 64;
  for (int i = tid; i < 64 * 32; i += 256) {
    const int k = i >> 5, e = i & 31;
    ws[k * PITCH + e] = e < RSC ? w[(kbase + k) * RSC + e] : from_f32<T>(0.f);
  }
  const int grp = tid & 7, slot = tid >> 3;
  const int pixels = g.N * g.P * g.Q;  // < 2^24 (checked by the launcher)
  const int H = g.H, W = g.W, cstride = g.stride, pad = g.pad;
  // this thread's depth elements e = grp + 8u of each of its four pixels
  int er[4], es[4], ec[4];
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int e = grp + 8 * u < RSC ? grp + 8 * u : RSC - 1;
    const int tap = e / C;
    ec[u] = e - tap * C; er[u] = tap / 3 - pad; es[u] = tap % 3 - pad;
  }
#pragma unroll
  for (int i = 0; i < PPT; ++i) {
    const int m = blockIdx.x * (32 * PPT) + slot + 32 * i;
    const uint32_t mm = m < pixels ? (uint32_t)m : 0u;
    const uint32_t n = divPQ.div(mm), rem = mm - n * divPQ.d;
    const uint32_t p = divQ.div(rem), q = rem - p * divQ.d;
    const int ih0 = (int)p * cstride, iw0 = (int)q * cstride, nbase = (int)n * H;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int ih = ih0 + er[u], iw = iw0 + es[u];
      const bool ok = ih >= 0 && ih < H && iw >= 0 && iw < W && grp + 8 * u < RSC;
      const T v = x[ok ? ((nbase + ih) * W + iw) * C + ec[u] : 0];
      xs[(slot + 32 * i) * PITCH + grp + 8 * u] = ok ? v : from_f32<T>(0.f);
    }
  }
  __syncthreads();
  // lane group g owns depth elements [16g, 16g + 16) of both operands (first MFMA: its first eight, second: the rest)
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1, hg = lane >> 5, l32 = lane & 31;
  const FV b0 = *reinterpret_cast<const FV*>(&ws[(wn * 32 + l32) * PITCH + hg * 16]);
  const FV b1 = *reinterpret_cast<const FV*>(&ws[(wn * 32 + l32) * PITCH + hg * 16 + 8]);
  v16f acc[2];
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const T* ap = &xs[(wm * 64 + i * 32 + l32) * PITCH + hg * 16];
    const FV a0 = *reinterpret_cast<const FV*>(ap);
    const FV a1 = *reinterpret_cast<const FV*>(ap + 8);
    v16f c;
#pragma unroll
    for (int e = 0; e < 16; ++e) c[e] = 0.f;
    c = StemMma<T>::run(a0, b0, c);
    acc[i] = StemMma<T>::run(a1, b1, c);
  }
  // epilogue: the 64 rows of one wavefront pair at a time through LDS as fp32 [64][64 + 4]
  constexpr int EP_PITCH = 64 + 4;
  float ss[8], qq[8];  // (channel sums: not used here)
#pragma unroll
  for (int k = 0; k < 8; ++k) { ss[k] = 0.f; qq[k] = 0.f; }
#pragma unroll
  for (int u = 0; u < 2; ++u) {
    __syncthreads();
    if (wm == u) {
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e)
          ep[(i * 32 + 8 * (e >> 2) + 4 * hg + (e & 3)) * EP_PITCH + wn * 32 + l32] = acc[i][e];
    }
    __syncthreads();
    auto rowoff = [&](int row) -> int64_t {
      const int64_t m = (int64_t)blockIdx.x * 128 + u * 64 + row;
      return m < pixels ? m * g.K : -1;
    };
    epi_store_pass<T, 64, 64, true, false, false>(ep, tid, kbase, bias, (const T*)nullptr, (const uint8_t*)nullptr, out, relu,
                                                  rowoff, ss, qq);
  }
}

// Weight gradient for few input channels (the network stem):  dw[k][e] = sum over pixels of dz[px][k] * col[px][e],
// e = (tap, c) < 36, k <= 64.  HBM-bound on reading dz once.  A block reduces a fixed chunk of pixels in tiles of 64:
// the dz tile [64][64] and the im2col tile [64][R*S*C] are staged in LDS as fp32 (two stages; the next tile's global
// loads are issued before the MFMAs of the current one).  Each wavefront multiplies 16 of the 64 pixels with fp32
// 32x32x2 MFMAs (rows k, columns e); the four partial sums are added in wavefront order through LDS.
template <class T>
__global__ void __launch_bounds__(256) conv_wgrad_smallc_kernel(const T* __restrict__ x, const T* __restrict__ dz,
                                                                float* __restrict__ partial, ConvGeom g, int chunk,
                                                                FastDiv divQ, FastDiv divPQ) {
  typedef __attribute__((ext_vector_type(16))) float v16f;
  constexpr int DP = 68, XP = 37;                          // LDS row pitches in floats
  constexpr int NX = (64 * SMALLC_MAX + 255) / 256;        // im2col elements per thread and tile
  constexpr int EV = 16 / (int)sizeof(T), CPP = 64 / EV;   // elements per 16-byte chunk, chunks per dz row
  constexpr int DCH = 64 * CPP / 256;                      // dz chunks per thread and tile
  __shared__ __attribute__((aligned(16))) float dzs[2][64 * DP];
  __shared__ float xs[2][64 * XP];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, hg = lane >> 5, l32 = lane & 31;
  const int K = g.K, C = g.C, H = g.H, W = g.W, rsc = g.R * g.S * g.C, cstride = g.stride;
  const int pixels = g.N * g.P * g.Q;
  const int m0 = blockIdx.x * chunk;
  const int m1 = m0 + chunk < pixels ? m0 + chunk : pixels;
  const int nt = m1 > m0 ? (m1 - m0 + 63) / 64 : 0;

  // tile-independent part of this thread's im2col elements: pixel row, filter offset, channel
  int xpx[NX], xdy[NX], xdx[NX], xc[NX], xdst[NX];
#pragma unroll
  for (int it = 0; it < NX; ++it) {
    const int i = tid + it * 256;
    const bool on = i < 64 * rsc;
    const int px = on ? i / rsc : 0, e = on ? i - px * rsc : 0;
    const int c = e % C, tap = e / C, s = tap % g.S, r = tap / g.S;
    xpx[it] = on ? px : -1; xdy[it] = r - g.pad; xdx[it] = s - g.pad; xc[it] = c; xdst[it] = px * XP + e;
  }
  Chunk rd[DCH];
  float rx[NX];
  unsigned dmask = 0u, xmask = 0u;
  // loads are unconditional (clamped addresses); what lies outside is zeroed when written to LDS
  auto gload = [&](int t) {
    const int mt = m0 + t * 64;
    unsigned dm = 0u, xm = 0u;
#pragma unroll
    for (int i = 0; i < DCH; ++i) {
      const int id = tid + i * 256, px = id / CPP, kv = id - px * CPP;
      const bool ok = mt + px < m1 && kv * EV < K;
      rd[i] = *reinterpret_cast<const Chunk*>(dz + (int64_t)(ok ? mt + px : m0) * K + (ok ? kv * EV : 0));
      dm |= ok ? (1u << i) : 0u;
    }
#pragma unroll
    for (int it = 0; it < NX; ++it) {
      const int m = mt + xpx[it];
      bool ok = xpx[it] >= 0 && m < m1;
      const uint32_t mm = ok ? (uint32_t)m : (uint32_t)m0;
      const uint32_t n_ = divPQ.div(mm), rem = mm - n_ * divPQ.d;
      const uint32_t p_ = divQ.div(rem), q_ = rem - p_ * divQ.d;
      const int ih = (int)p_ * cstride + xdy[it], iw = (int)q_ * cstride + xdx[it];
      ok = ok && ih >= 0 && ih < H && iw >= 0 && iw < W;
      const int64_t off = ok ? (((int64_t)n_ * H + ih) * W + iw) * C + xc[it] : 0;
      rx[it] = to_f32(x[off]);
      xm |= ok ? (1u << it) : 0u;
    }
    dmask = dm; xmask = xm;
  };
  auto sstore = [&](int stage) {
#pragma unroll
    for (int i = 0; i < DCH; ++i) {
      const int id = tid + i * 256, px = id / CPP, kv = id - px * CPP;
      const Chunk c = ((dmask >> i) & 1u) ? rd[i] : zero_chunk();
      float* dst = &dzs[stage][px * DP + kv * EV];
      if constexpr (sizeof(T) == 4) {
        *reinterpret_cast<Chunk*>(dst) = c;
      } else {
        const Vec<T, EV> v = __builtin_bit_cast(Vec<T, EV>, c);
        float f[EV];
#pragma unroll
        for (int k = 0; k < EV; ++k) f[k] = to_f32(v.v[k]);
#pragma unroll
        for (int k = 0; k < EV; k += 4) {
          typedef __attribute__((ext_vector_type(4))) float v4f;
          v4f o = {f[k], f[k + 1], f[k + 2], f[k + 3]};
          *reinterpret_cast<v4f*>(dst + k) = o;
        }
      }
    }
#pragma unroll
    for (int it = 0; it < NX; ++it)
      if (xpx[it] >= 0) xs[stage][xdst[it]] = ((xmask >> it) & 1u) ? rx[it] : 0.f;
  };

  v16f acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
  const bool two_m = K > 32, two_n = rsc > 32;
  const int e0 = l32 < rsc ? l32 : rsc - 1, e1 = 32 + l32 < rsc ? 32 + l32 : rsc - 1;
  const float z0 = l32 < rsc ? 1.f : 0.f, z1 = 32 + l32 < rsc ? 1.f : 0.f;

  if (nt > 0) { gload(0); sstore(0); }
  __syncthreads();
  for (int t = 0; t < nt; ++t) {
    const int stage = t & 1;
    if (t + 1 < nt) gload(t + 1);
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int px = 16 * wave + 8 * hg + u;
      const float a0 = dzs[stage][px * DP + l32];
      const float b0 = xs[stage][px * XP + e0] * z0;
      acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b0, acc[0][0], 0, 0, 0);
      float a1 = 0.f;
      if (two_m) {
        a1 = dzs[stage][px * DP + 32 + l32];
        acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b0, acc[1][0], 0, 0, 0);
      }
      if (two_n) {
        const float b1 = xs[stage][px * XP + e1] * z1;
        acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b1, acc[0][1], 0, 0, 0);
        if (two_m) acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b1, acc[1][1], 0, 0, 0);
      }
    }
    if (t + 1 < nt) sstore(stage ^ 1);
    __syncthreads();
  }

  // the four wavefronts' sums, added in wavefront order: red[k][e], pitch 65
  float* red = &dzs[0][0];
#pragma unroll 1
  for (int w = 0; w < 4; ++w) {
    if (wave == w) {
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
          for (int e = 0; e < 16; ++e) {
            const int idx = (i * 32 + 8 * (e >> 2) + 4 * hg + (e & 3)) * 65 + j * 32 + l32;
            red[idx] = w == 0 ? acc[i][j][e] : red[idx] + acc[i][j][e];
          }
    }
    __syncthreads();
  }
  for (int o = tid; o < K * rsc; o += 256) {
    const int k = o / rsc, e = o - k * rsc;
    partial[((int64_t)blockIdx.x * K + k) * rsc + e] = red[k * 65 + e];
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

bool conv_smallc_fwd_ok(const ConvGeom& g) {
  return g.C <= 4 && g.R == 3 && g.S == 3 && g.K % 8 == 0 && (int64_t)g.N * g.P * g.Q < (1 << 24) &&
         (int64_t)g.N * g.H * g.W * g.C < ((int64_t)1 << 31);
}
bool conv_smallc_wgrad_ok(const ConvGeom& g) {
  return g.C <= 4 && g.R * g.S * g.C <= SMALLC_MAX && g.K <= 64 && g.K % 8 == 0 && (int64_t)g.N * g.P * g.Q < (1 << 24) &&
         (int64_t)g.N * g.H * g.W * g.C < ((int64_t)1 << 31);
}
int conv_smallc_wgrad_splits(const ConvGeom& g) {
  const int64_t pixels = (int64_t)g.N * g.P * g.Q;
  int64_t b = (pixels + 255) / 256;
  return (int)(b < 1 ? 1 : (b > 1024 ? 1024 : b));
}

template <class T>
static void launch_fwd_smallc_t(hipStream_t st, const void* x, const void* w, const float* bias, void* out, const ConvGeom& g,
                                int relu) {
  dim3 grid(ceil_div((int64_t)g.N * g.P * g.Q, 128), ceil_div(g.K, 64)), block(256);
  const FastDiv dq = make_fastdiv((uint32_t)g.Q), dpq = make_fastdiv((uint32_t)(g.P * g.Q));
  if constexpr (sizeof(T) == 2) {
    if (g.K % 64 == 0 && g.C <= 3) {  // 16-bit modes: on the matrix cores
      switch (g.C) {
        case 1: OSEQ_LAUNCH((conv_fwd_smallc_mfma_kernel<T, 1>), grid, block, 0, st, (const T*)x, (const T*)w, bias, (T*)out, g, relu, dq, dpq); break;
        case 2: OSEQ_LAUNCH((conv_fwd_smallc_mfma_kernel<T, 2>), grid, block, 0, st, (const T*)x, (const T*)w, bias, (T*)out, g, relu, dq, dpq); break;
        default: OSEQ_LAUNCH((conv_fwd_smallc_mfma_kernel<T, 3>), grid, block, 0, st, (const T*)x, (const T*)w, bias, (T*)out, g, relu, dq, dpq); break;
      }
      return;
    }
  }
  switch (g.C) {
    case 1: OSEQ_LAUNCH((conv_fwd_smallc_kernel<T, 1>), grid, block, 0, st, (const T*)x, (const T*)w, bias, (T*)out, g, relu, dq, dpq); break;
    case 2: OSEQ_LAUNCH((conv_fwd_smallc_kernel<T, 2>), grid, block, 0, st, (const T*)x, (const T*)w, bias, (T*)out, g, relu, dq, dpq); break;
    case 3: OSEQ_LAUNCH((conv_fwd_smallc_kernel<T, 3>), grid, block, 0, st, (const T*)x, (const T*)w, bias, (T*)out, g, relu, dq, dpq); break;
    default: OSEQ_LAUNCH((conv_fwd_smallc_kernel<T, 4>), grid, block, 0, st, (const T*)x, (const T*)w, bias, (T*)out, g, relu, dq, dpq); break;
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
  const FastDiv dq = make_fastdiv((uint32_t)g.Q), dpq = make_fastdiv((uint32_t)(g.P * g.Q));
  if (dt == DT_F32) OSEQ_LAUNCH(conv_wgrad_smallc_kernel<float>, grid, block, 0, st, (const float*)x, (const float*)dz, dst, g, chunk, dq, dpq);
  else if (dt == DT_BF16) OSEQ_LAUNCH(conv_wgrad_smallc_kernel<bf16_t>, grid, block, 0, st, (const bf16_t*)x, (const bf16_t*)dz, dst, g, chunk, dq, dpq);
  else OSEQ_LAUNCH(conv_wgrad_smallc_kernel<f16_t>, grid, block, 0, st, (const f16_t*)x, (const f16_t*)dz, dst, g, chunk, dq, dpq);
  if (splits > 1) {
    const int64_t n = (int64_t)g.K * g.R * g.S * g.C;
    OSEQ_LAUNCH(wave_reduce_kernel, dim3(ceil_div(n, 4)), dim3(256), 0, st, partial, dw, n, splits);
  }
}

void launch_conv_fwd_direct(hipStream_t st, int dt, const void* x, const void* w, const float* bias, void* out,
                            const ConvGeom& g, int relu) {
  const int64_t total = (int64_t)g.N * g.P * g.Q * g.K;
  dim3 grid(ceil_div(total, 256)), block(256);
  if (dt == DT_F32) OSEQ_LAUNCH(conv_fwd_direct_kernel<float>, grid, block, 0, st, (const float*)x, (const float*)w, bias, (float*)out, g, relu);
  else if (dt == DT_BF16) OSEQ_LAUNCH(conv_fwd_direct_kernel<bf16_t>, grid, block, 0, st, (const bf16_t*)x, (const bf16_t*)w, bias, (bf16_t*)out, g, relu);
  else OSEQ_LAUNCH(conv_fwd_direct_kernel<f16_t>, grid, block, 0, st, (const f16_t*)x, (const f16_t*)w, bias, (f16_t*)out, g, relu);
}

void launch_conv_dgrad_direct(hipStream_t st, int dt, const void* dz, const void* w, const void* addend, void* dx,
                              const ConvGeom& g) {
  const int64_t total = (int64_t)g.N * g.H * g.W * g.C;
  dim3 grid(ceil_div(total, 256)), block(256);
  if (dt == DT_F32) OSEQ_LAUNCH(conv_dgrad_direct_kernel<float>, grid, block, 0, st, (const float*)dz, (const float*)w, (const float*)addend, (float*)dx, g);
  else if (dt == DT_BF16) OSEQ_LAUNCH(conv_dgrad_direct_kernel<bf16_t>, grid, block, 0, st, (const bf16_t*)dz, (const bf16_t*)w, (const bf16_t*)addend, (bf16_t*)dx, g);
  else OSEQ_LAUNCH(conv_dgrad_direct_kernel<f16_t>, grid, block, 0, st, (const f16_t*)dz, (const f16_t*)w, (const f16_t*)addend, (f16_t*)dx, g);
}

void launch_conv_wgrad_direct(hipStream_t st, int dt, const void* x, const void* dz, float* dw, float* partial, int splits,
                              const ConvGeom& g) {
  const int64_t outputs = (int64_t)g.K * g.R * g.S * g.C;
  const int64_t pixels = (int64_t)g.N * g.P * g.Q;
  const int64_t chunk = (pixels + splits - 1) / splits;
  float* dst = splits > 1 ? partial : dw;
  dim3 grid(ceil_div(outputs, 256), splits), block(256);
  if (dt == DT_F32) OSEQ_LAUNCH(conv_wgrad_direct_kernel<float>, grid, block, 0, st, (const float*)x, (const float*)dz, dst, g, chunk);
  else if (dt == DT_BF16) OSEQ_LAUNCH(conv_wgrad_direct_kernel<bf16_t>, grid, block, 0, st, (const bf16_t*)x, (const bf16_t*)dz, dst, g, chunk);
  else OSEQ_LAUNCH(conv_wgrad_direct_kernel<f16_t>, grid, block, 0, st, (const f16_t*)x, (const f16_t*)dz, dst, g, chunk);
  if (splits > 1)
    OSEQ_LAUNCH(splitk_reduce_kernel, dim3(ceil_div(outputs, 256)), dim3(256), 0, st, partial, dw, outputs, splits);
}

}  // namespace oseq
