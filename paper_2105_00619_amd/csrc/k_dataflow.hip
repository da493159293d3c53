// Image data-flow kernels (paper, Section "Image Data-flow Optimization"): Algorithms "Encode", "Decode" and
// "Loss-less Forced Encoding" on the device.
//
// With base 256 the number of a position is, in memory, the bytes of its images side by side: image i of a group is
// byte i of the position's little-endian words.  Encode and Decode are therefore byte transposes between
// [image][position] and [position][image], bound by HBM traffic.  One block handles 2048 positions of one group (1024
// where that fills an image's last block better): a thread reads 8 consecutive positions of every image with one 8-byte load (a wavefront reads 512 contiguous bytes
// per image), transposes 8 x 8 bytes with byte permutes, and the words travel through LDS so that the other side is
// accessed as 16 contiguous bytes per lane as well.  Decode can apply pixel * scale[c] + shift[c] and the cast to the
// network's storage type on the way out, which makes it the first layer of a network.
//
// The loss-less form has 7-bit digits that straddle word boundaries; its kernels build the words with shifts, four
// positions per thread.
//
// Inputs that do not meet the fast kernels' shape and alignment needs take one-position-per-thread kernels.
#include "dev_common.h"

namespace oseq {

static constexpr int g_df_threads = 0;  // compile-time constant: 0 = chosen from the image size

namespace {

constexpr int DF_POS = 8;  // positions per thread; a block of n threads (256, or 128 for short images) handles 8 n positions

struct DfNorm { float scale[16]; float shift[16]; int channels; };

// byte k of the result = byte sel_k of the pair: 0..3 from `lo`, 4..7 from `hi`
__device__ __forceinline__ uint32_t bperm(uint32_t hi, uint32_t lo, uint32_t sel) { return __builtin_amdgcn_perm(hi, lo, sel); }

// 4 x 4 byte transpose: byte j of a_i becomes byte i of b_j
__device__ __forceinline__ void t4x4(uint32_t a0, uint32_t a1, uint32_t a2, uint32_t a3, uint32_t& b0, uint32_t& b1,
                                     uint32_t& b2, uint32_t& b3) {
  const uint32_t t0 = bperm(a1, a0, 0x05010400u);  // a0.0 a1.0 a0.1 a1.1
  const uint32_t t1 = bperm(a1, a0, 0x07030602u);  // a0.2 a1.2 a0.3 a1.3
  const uint32_t t2 = bperm(a3, a2, 0x05010400u);
  const uint32_t t3 = bperm(a3, a2, 0x07030602u);
  b0 = bperm(t2, t0, 0x05040100u);
  b1 = bperm(t2, t0, 0x07060302u);
  b2 = bperm(t3, t1, 0x05040100u);
  b3 = bperm(t3, t1, 0x07060302u);
}

// 8 x 8 byte transpose of rows (lo = bytes 0..3, hi = bytes 4..7): byte j of row i becomes byte i of row j
__device__ __forceinline__ void t8x8(const uint32_t* ilo, const uint32_t* ihi, uint32_t* olo, uint32_t* ohi) {
  t4x4(ilo[0], ilo[1], ilo[2], ilo[3], olo[0], olo[1], olo[2], olo[3]);
  t4x4(ihi[0], ihi[1], ihi[2], ihi[3], olo[4], olo[5], olo[6], olo[7]);
  t4x4(ilo[4], ilo[5], ilo[6], ilo[7], ohi[0], ohi[1], ohi[2], ohi[3]);
  t4x4(ihi[4], ihi[5], ihi[6], ihi[7], ohi[4], ohi[5], ohi[6], ohi[7]);
}

// LDS slot of 16-byte chunk q of a block's words: one slot of padding after every 16, so that the threads' 64- or
// 128-byte pieces and the lane-contiguous accesses are both free of bank conflicts
__device__ __forceinline__ int df_slot(int q) { return q + (q >> 4); }

// dynamic LDS of a block of nthr threads: its 4 W chunks per thread plus the padding slots
inline size_t df_lds_bytes(int W, int nthr) { return (size_t)(nthr * 4 * W + nthr * 4 * W / 16) * 16; }

// ---- Encode: x [B][P] bytes -> a [G][P][W] words ---------------------------------------------------------------
template <int W>
__global__ __launch_bounds__(256) void encode_kernel(const uint8_t* __restrict__ x, uint4* __restrict__ a4, int z, int64_t P,
                                                     int64_t B, int tiles) {
  extern __shared__ uint4 buf[];
  const int tid = threadIdx.x, nthr = blockDim.x;
  const int tile_pos = nthr * DF_POS;
  const int64_t g = blockIdx.x / tiles;
  const int tile = blockIdx.x % tiles;
  const int64_t p0 = (int64_t)tile * tile_pos + tid * 8;
  const int64_t n0 = g * z;
  const int zg = (int)((B - n0) < (int64_t)z ? (B - n0) : (int64_t)z);
  uint32_t lo[8 * W], hi[8 * W];
#pragma unroll
  for (int i = 0; i < 8 * W; ++i) {
    uint2 v = make_uint2(0u, 0u);
    if (i < zg && p0 < P) v = *reinterpret_cast<const uint2*>(x + (n0 + i) * P + p0);
    lo[i] = v.x; hi[i] = v.y;
  }
  uint32_t wlo[W][8], whi[W][8];  // word w of position j
#pragma unroll
  for (int w = 0; w < W; ++w) t8x8(lo + 8 * w, hi + 8 * w, wlo[w], whi[w]);
  if (W == 1) {
#pragma unroll
    for (int c = 0; c < 4; ++c) buf[df_slot(tid * 4 + c)] = make_uint4(wlo[0][2 * c], whi[0][2 * c], wlo[0][2 * c + 1], whi[0][2 * c + 1]);
  } else {
#pragma unroll
    for (int c = 0; c < 8; ++c) buf[df_slot(tid * 8 + c)] = make_uint4(wlo[0][c], whi[0][c], wlo[W - 1][c], whi[W - 1][c]);
  }
  __syncthreads();
  uint4* dst = a4 + (g * P * W) / 2 + (int64_t)tile * (tile_pos / 2 * W);
#pragma unroll
  for (int m = 0; m < 4 * W; ++m) {
    const int q = tid + nthr * m;
    const int64_t pos = (int64_t)tile * tile_pos + (W == 1 ? 2 * q : q);
    if (pos < P) dst[q] = buf[df_slot(q)];
  }
}

// ---- Decode: a -> bytes, or -> pixel * scale + shift in T ------------------------------------------------------
template <class T>
__device__ __forceinline__ void store_pixels8(T* dst, uint32_t blo, uint32_t bhi, const float (&sc)[8], const float (&sh)[8]) {
  float v[8];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    v[j] = __fmaf_rn((float)((blo >> (8 * j)) & 0xffu), sc[j], sh[j]);
    v[4 + j] = __fmaf_rn((float)((bhi >> (8 * j)) & 0xffu), sc[4 + j], sh[4 + j]);
  }
  Vec<T, 4> t0, t1;
#pragma unroll
  for (int j = 0; j < 4; ++j) { t0.v[j] = from_f32<T>(v[j]); t1.v[j] = from_f32<T>(v[4 + j]); }
  *reinterpret_cast<Vec<T, 4>*>(dst) = t0;
  *reinterpret_cast<Vec<T, 4>*>(dst + 4) = t1;
}

// T = uint8_t: plain Decode; else the normalised form
template <int W, class T>
__global__ __launch_bounds__(256) void decode_kernel(const uint4* __restrict__ a4, T* __restrict__ out, int z, int64_t P,
                                                     int64_t B, int tiles, DfNorm nm) {
  constexpr bool RAW = sizeof(T) == 1;
  extern __shared__ uint4 buf[];
  __shared__ float s_scale[16], s_shift[16];
  const int tid = threadIdx.x, nthr = blockDim.x;
  const int tile_pos = nthr * DF_POS;
  const int64_t g = blockIdx.x / tiles;
  const int tile = blockIdx.x % tiles;
  const int64_t p0 = (int64_t)tile * tile_pos + tid * 8;
  const int64_t n0 = g * z;
  const int zg = (int)((B - n0) < (int64_t)z ? (B - n0) : (int64_t)z);
  const uint4* src = a4 + (g * P * W) / 2 + (int64_t)tile * (tile_pos / 2 * W);
  uint4 ch[4 * W];
#pragma unroll
  for (int m = 0; m < 4 * W; ++m) {
    const int q = tid + nthr * m;
    const int64_t pos = (int64_t)tile * tile_pos + (W == 1 ? 2 * q : q);
    ch[m] = make_uint4(0u, 0u, 0u, 0u);
    if (pos < P) ch[m] = src[q];
  }
#pragma unroll
  for (int m = 0; m < 4 * W; ++m) buf[df_slot(tid + nthr * m)] = ch[m];
  if (!RAW && tid < 16) { s_scale[tid] = nm.scale[tid]; s_shift[tid] = nm.shift[tid]; }
  __syncthreads();
  if (p0 >= P) return;
  uint32_t wlo[W][8], whi[W][8];
  if (W == 1) {
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const uint4 v = buf[df_slot(tid * 4 + c)];
      wlo[0][2 * c] = v.x; whi[0][2 * c] = v.y; wlo[0][2 * c + 1] = v.z; whi[0][2 * c + 1] = v.w;
    }
  } else {
#pragma unroll
    for (int c = 0; c < 8; ++c) {
      const uint4 v = buf[df_slot(tid * 8 + c)];
      wlo[0][c] = v.x; whi[0][c] = v.y; wlo[W - 1][c] = v.z; whi[W - 1][c] = v.w;
    }
  }
  uint32_t lo[8 * W], hi[8 * W];  // image i: its 8 positions
#pragma unroll
  for (int w = 0; w < W; ++w) t8x8(wlo[w], whi[w], lo + 8 * w, hi + 8 * w);
  if constexpr (RAW) {
#pragma unroll
    for (int i = 0; i < 8 * W; ++i)
      if (i < zg) *reinterpret_cast<uint2*>(out + (n0 + i) * P + p0) = make_uint2(lo[i], hi[i]);
  } else {
    float sc[8], sh[8];
    const int C = nm.channels;
    int c = (int)(p0 % C);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      sc[j] = s_scale[c]; sh[j] = s_shift[c];
      c = c + 1 == C ? 0 : c + 1;
    }
#pragma unroll
    for (int i = 0; i < 8 * W; ++i)
      if (i < zg) store_pixels8<T>(out + (n0 + i) * P + p0, lo[i], hi[i], sc, sh);
  }
}

// ---- any shape and alignment: one position per thread ---------------------------------------------------------------
template <int W>
__global__ __launch_bounds__(256) void encode_pos_kernel(const uint8_t* __restrict__ x, uint64_t* __restrict__ a, int z,
                                                         int64_t P, int64_t B, int64_t total) {
  const int64_t u = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (u >= total) return;
  const int64_t g = u / P, p = u % P, n0 = g * z;
  const int zg = (int)((B - n0) < (int64_t)z ? (B - n0) : (int64_t)z);
  uint64_t w[W];
#pragma unroll
  for (int k = 0; k < W; ++k) w[k] = 0;
#pragma unroll
  for (int i = 0; i < 8 * W; ++i)
    if (i < zg) w[i / 8] |= (uint64_t)x[(n0 + i) * P + p] << (8 * (i % 8));
#pragma unroll
  for (int k = 0; k < W; ++k) a[u * W + k] = w[k];
}

template <int W, class T>
__global__ __launch_bounds__(256) void decode_pos_kernel(const uint64_t* __restrict__ a, T* __restrict__ out, int z, int64_t P,
                                                         int64_t B, int64_t total, DfNorm nm) {
  constexpr bool RAW = sizeof(T) == 1;
  const int64_t u = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (u >= total) return;
  const int64_t g = u / P, p = u % P, n0 = g * z;
  const int zg = (int)((B - n0) < (int64_t)z ? (B - n0) : (int64_t)z);
  uint64_t w[W];
#pragma unroll
  for (int k = 0; k < W; ++k) w[k] = a[u * W + k];
  float sc = 0.f, sh = 0.f;
  if (!RAW) {
    const int c = (int)(p % nm.channels);
#pragma unroll
    for (int k = 0; k < 16; ++k)
      if (k == c) { sc = nm.scale[k]; sh = nm.shift[k]; }
  }
#pragma unroll
  for (int i = 0; i < 8 * W; ++i) {
    if (i >= zg) continue;
    const uint32_t b = (uint32_t)(w[i / 8] >> (8 * (i % 8))) & 0xffu;
    if constexpr (RAW) out[(n0 + i) * P + p] = (T)b;
    else out[(n0 + i) * P + p] = from_f32<T>(__fmaf_rn((float)b, sc, sh));
  }
}

// ---- loss-less form: 7-bit digits, parities apart ----------------------------------------------------------
// digit i sits at bits 7 i .. 7 i + 6 of the number; L words hold min(32, 64 L / 7) digits
template <int L>
constexpr int ll_zmax() { return 64 * L / 7 < 32 ? 64 * L / 7 : 32; }

template <int L, int VEC>
__global__ __launch_bounds__(256) void encode_lossless_kernel(const uint8_t* __restrict__ x, uint64_t* __restrict__ a,
                                                              uint32_t* __restrict__ o, int z, int64_t P, int64_t B,
                                                              int64_t total) {
  const int64_t u = (int64_t)blockIdx.x * 256 + threadIdx.x;  // unit = VEC consecutive positions of one group
  if (u >= total) return;
  const int64_t PV = P / VEC;
  const int64_t g = u / PV, p = (u % PV) * VEC, n0 = g * z;
  const int zg = (int)((B - n0) < (int64_t)z ? (B - n0) : (int64_t)z);
  uint64_t limb[VEC][L];
  uint32_t off[VEC];
#pragma unroll
  for (int q = 0; q < VEC; ++q) {
    off[q] = 0;
#pragma unroll
    for (int l = 0; l < L; ++l) limb[q][l] = 0;
  }
  uint32_t px[ll_zmax<L>()];
#pragma unroll
  for (int i = 0; i < ll_zmax<L>(); ++i) {
    px[i] = 0;
    if (i < zg) {
      if (VEC == 4) px[i] = *reinterpret_cast<const uint32_t*>(x + (n0 + i) * P + p);
      else px[i] = x[(n0 + i) * P + p];
    }
  }
#pragma unroll
  for (int i = 0; i < ll_zmax<L>(); ++i) {
    const int bit = 7 * i, lw = bit / 64, sft = bit % 64;
#pragma unroll
    for (int q = 0; q < VEC; ++q) {
      const uint32_t b = (px[i] >> (8 * q)) & 0xffu;
      off[q] |= (b & 1u) << i;
      const uint64_t d = b >> 1;
      limb[q][lw] |= d << sft;
      if (sft > 57 && lw + 1 < L) limb[q][lw + 1] |= d >> (64 - sft);
    }
  }
  const int64_t e = g * P + p;
  if (VEC == 4) {
    uint4* dst = reinterpret_cast<uint4*>(a + e * L);
#pragma unroll
    for (int k = 0; k < 2 * L; ++k) {  // 4 positions x L words = 2 L chunks of two words
      const int i0 = 2 * k, i1 = 2 * k + 1;
      const uint64_t w0 = limb[i0 / L][i0 % L], w1 = limb[i1 / L][i1 % L];
      dst[k] = make_uint4((uint32_t)w0, (uint32_t)(w0 >> 32), (uint32_t)w1, (uint32_t)(w1 >> 32));
    }
    *reinterpret_cast<uint4*>(o + e) = make_uint4(off[0], off[VEC > 1 ? 1 : 0], off[VEC > 2 ? 2 : 0], off[VEC > 3 ? 3 : 0]);
  } else {
#pragma unroll
    for (int l = 0; l < L; ++l) a[e * L + l] = limb[0][l];
    o[e] = off[0];
  }
}

template <int L, int VEC>
__global__ __launch_bounds__(256) void decode_lossless_kernel(const uint64_t* __restrict__ a, const uint32_t* __restrict__ o,
                                                              uint8_t* __restrict__ x, int z, int64_t P, int64_t B,
                                                              int64_t total) {
  const int64_t u = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (u >= total) return;
  const int64_t PV = P / VEC;
  const int64_t g = u / PV, p = (u % PV) * VEC, n0 = g * z;
  const int zg = (int)((B - n0) < (int64_t)z ? (B - n0) : (int64_t)z);
  const int64_t e = g * P + p;
  uint64_t limb[VEC][L];
  uint32_t off[VEC];
  if (VEC == 4) {
    const uint4* src = reinterpret_cast<const uint4*>(a + e * L);
#pragma unroll
    for (int k = 0; k < 2 * L; ++k) {
      const uint4 v = src[k];
      const int i0 = 2 * k, i1 = 2 * k + 1;
      limb[i0 / L][i0 % L] = (uint64_t)v.x | ((uint64_t)v.y << 32);
      limb[i1 / L][i1 % L] = (uint64_t)v.z | ((uint64_t)v.w << 32);
    }
    const uint4 ov = *reinterpret_cast<const uint4*>(o + e);
    off[0] = ov.x; off[VEC > 1 ? 1 : 0] = ov.y; off[VEC > 2 ? 2 : 0] = ov.z; off[VEC > 3 ? 3 : 0] = ov.w;
  } else {
#pragma unroll
    for (int l = 0; l < L; ++l) limb[0][l] = a[e * L + l];
    off[0] = o[e];
  }
#pragma unroll
  for (int i = 0; i < ll_zmax<L>(); ++i) {
    if (i >= zg) continue;
    const int bit = 7 * i, lw = bit / 64, sft = bit % 64;
    uint32_t packed = 0;
#pragma unroll
    for (int q = 0; q < VEC; ++q) {
      uint64_t d = limb[q][lw] >> sft;
      if (sft > 57 && lw + 1 < L) d |= limb[q][lw + 1] << (64 - sft);
      const uint32_t b = 2u * ((uint32_t)d & 127u) + ((off[q] >> i) & 1u);
      packed |= b << (8 * q);
    }
    if (VEC == 4) *reinterpret_cast<uint32_t*>(x + (n0 + i) * P + p) = packed;
    else x[(n0 + i) * P + p] = (uint8_t)packed;
  }
}

// 256 threads per block, or 128 where that leaves fewer idle threads in an image's last block (a 32 x 32 x 3 image is
// one and a half blocks of 256 threads, and three full ones of 128)
int df_threads(int64_t P) {
  if (g_df_threads == 128 || g_df_threads == 256) return g_df_threads;
  const int64_t idle256 = (P + 2047) / 2048 * 2048 - P, idle128 = (P + 1023) / 1024 * 1024 - P;
  return idle128 < idle256 ? 128 : 256;
}

bool aligned(const void* p, size_t n) { return (reinterpret_cast<uintptr_t>(p) & (n - 1)) == 0; }

DfNorm make_norm(int channels, const float* scale, const float* shift) {
  DfNorm nm{};
  nm.channels = channels;
  for (int c = 0; c < 16; ++c) { nm.scale[c] = c < channels ? scale[c] : 0.f; nm.shift[c] = c < channels ? shift[c] : 0.f; }
  return nm;
}

template <class T>
void launch_decode_t(hipStream_t st, const uint64_t* a, int64_t B, int64_t P, int z, T* out, const DfNorm& nm) {
  const int64_t G = (B + z - 1) / z;
  const int W = (z + 7) / 8;
  if (P % 8 == 0 && aligned(a, 16) && aligned(out, sizeof(T) == 1 ? 8 : 16)) {
    const int nthr = df_threads(P);
    const int tiles = (int)((P + nthr * DF_POS - 1) / (nthr * DF_POS));
    const dim3 grid((unsigned)(G * tiles)), block(nthr);
    if (W == 1) OSEQ_LAUNCH((decode_kernel<1, T>), grid, block, df_lds_bytes(1, nthr), st, (const uint4*)a, out, z, P, B, tiles, nm);
    else OSEQ_LAUNCH((decode_kernel<2, T>), grid, block, df_lds_bytes(2, nthr), st, (const uint4*)a, out, z, P, B, tiles, nm);
  } else {
    const int64_t total = G * P;
    const dim3 grid((unsigned)((total + 255) / 256)), block(256);
    if (W == 1) OSEQ_LAUNCH((decode_pos_kernel<1, T>), grid, block, 0, st, a, out, z, P, B, total, nm);
    else OSEQ_LAUNCH((decode_pos_kernel<2, T>), grid, block, 0, st, a, out, z, P, B, total, nm);
  }
}

}  // namespace

void launch_encode(hipStream_t st, const uint8_t* x, int64_t B, int64_t P, int z, uint64_t* a) {
  if (B <= 0 || P <= 0) return;
  const int64_t G = (B + z - 1) / z;
  const int W = (z + 7) / 8;
  if (P % 8 == 0 && aligned(x, 8) && aligned(a, 16)) {
    const int nthr = df_threads(P);
    const int tiles = (int)((P + nthr * DF_POS - 1) / (nthr * DF_POS));
    const dim3 grid((unsigned)(G * tiles)), block(nthr);
    if (W == 1) OSEQ_LAUNCH(encode_kernel<1>, grid, block, df_lds_bytes(1, nthr), st, x, (uint4*)a, z, P, B, tiles);
    else OSEQ_LAUNCH(encode_kernel<2>, grid, block, df_lds_bytes(2, nthr), st, x, (uint4*)a, z, P, B, tiles);
  } else {
    const int64_t total = G * P;
    const dim3 grid((unsigned)((total + 255) / 256)), block(256);
    if (W == 1) OSEQ_LAUNCH(encode_pos_kernel<1>, grid, block, 0, st, x, a, z, P, B, total);
    else OSEQ_LAUNCH(encode_pos_kernel<2>, grid, block, 0, st, x, a, z, P, B, total);
  }
}

void launch_decode(hipStream_t st, const uint64_t* a, int64_t B, int64_t P, int z, uint8_t* x) {
  if (B <= 0 || P <= 0) return;
  launch_decode_t<uint8_t>(st, a, B, P, z, x, DfNorm{});
}

void launch_decode_cast(hipStream_t st, int dt, const uint64_t* a, int64_t B, int64_t P, int z, int channels,
                        const float* scale, const float* shift, void* out) {
  if (B <= 0 || P <= 0) return;
  const DfNorm nm = make_norm(channels, scale, shift);
  if (dt == DT_F32) launch_decode_t<float>(st, a, B, P, z, (float*)out, nm);
  else if (dt == DT_BF16) launch_decode_t<bf16_t>(st, a, B, P, z, (bf16_t*)out, nm);
  else launch_decode_t<f16_t>(st, a, B, P, z, (f16_t*)out, nm);
}

template <int L>
static void launch_ll_l(hipStream_t st, bool enc, const uint8_t* x, uint64_t* a, uint32_t* o, uint8_t* xo, int64_t B, int64_t P,
                        int z) {
  const int64_t G = (B + z - 1) / z;
  const bool fast = P % 4 == 0 && aligned(enc ? (const void*)x : (const void*)xo, 4) && aligned(a, 16) && aligned(o, 16);
  const int64_t total = fast ? G * (P / 4) : G * P;
  const dim3 grid((unsigned)((total + 255) / 256)), block(256);
  if (enc) {
    if (fast) OSEQ_LAUNCH((encode_lossless_kernel<L, 4>), grid, block, 0, st, x, a, o, z, P, B, total);
    else OSEQ_LAUNCH((encode_lossless_kernel<L, 1>), grid, block, 0, st, x, a, o, z, P, B, total);
  } else {
    if (fast) OSEQ_LAUNCH((decode_lossless_kernel<L, 4>), grid, block, 0, st, (const uint64_t*)a, (const uint32_t*)o, xo, z, P, B, total);
    else OSEQ_LAUNCH((decode_lossless_kernel<L, 1>), grid, block, 0, st, (const uint64_t*)a, (const uint32_t*)o, xo, z, P, B, total);
  }
}

static void launch_ll(hipStream_t st, bool enc, const uint8_t* x, uint64_t* a, uint32_t* o, uint8_t* xo, int64_t B, int64_t P,
                      int z) {
  if (B <= 0 || P <= 0) return;
  switch ((7 * z + 63) / 64) {
    case 1: launch_ll_l<1>(st, enc, x, a, o, xo, B, P, z); break;
    case 2: launch_ll_l<2>(st, enc, x, a, o, xo, B, P, z); break;
    case 3: launch_ll_l<3>(st, enc, x, a, o, xo, B, P, z); break;
    default: launch_ll_l<4>(st, enc, x, a, o, xo, B, P, z); break;
  }
}

void launch_encode_lossless(hipStream_t st, const uint8_t* x, int64_t B, int64_t P, int z, uint64_t* a, uint32_t* o) {
  launch_ll(st, true, x, a, o, nullptr, B, P, z);
}

void launch_decode_lossless(hipStream_t st, const uint64_t* a, const uint32_t* o, int64_t B, int64_t P, int z, uint8_t* x) {
  launch_ll(st, false, nullptr, const_cast<uint64_t*>(a), const_cast<uint32_t*>(o), x, B, P, z);
}

}  // namespace oseq
