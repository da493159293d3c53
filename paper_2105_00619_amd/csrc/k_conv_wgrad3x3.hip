// Weight gradient of 3x3, stride-1 convolutions on the matrix cores, all nine filter taps in one block.
//
//   dw[k][r][s][c] = sum over output pixels (n, p, q) of dz[n, p, q, k] * x[n, p + r - pad, q + s - pad, c]
//
// One block owns 64*MI output channels k, 64 input channels c, all nine taps, and a fixed range of pixel sub-tiles
// (blockIdx.z); the ranges are summed afterwards in order, so the result does not depend on scheduling.  A sub-tile is
// TI images x TR rows x TC columns of output pixels (at most CAP); its dz rows and the x positions it touches (the
// sub-tile plus a one-pixel halo, zero outside the image) are staged once in LDS, pixel-major as loaded, and serve
// all nine taps: a tap only shifts the x position that is paired with a dz pixel.  Compared with one tap per block
// this reads dz once instead of nine times and x about twice instead of nine times, which is what bounds the
// 16-bit kernel (the path from L2 to LDS), and it leaves nine MFMAs per operand fetch.
//
//   block = WGM x 2 wavefronts: wavefront (wm, wn) owns k rows [wm*32*MI, +32*MI) and c columns [wn*32, +32) of
//   every tap: MI x 9 accumulator tiles of 32x32.  64 output channels: 2 x 2 wavefronts, one per SIMD.  128 output
//   channels (16-bit modes): 4 x 2 wavefronts with MI = 1, two per SIMD (144 accumulator registers each), so that one
//   wavefront's LDS reads and address arithmetic run under the other's MFMAs: 256 -> 256 channels at 8 x 8, batch
//   4096, bf16: 481 us with 2 x 2 wavefronts of MI = 2, 326 us with 4 x 2 (the one-tap-per-block kernel: 479 us).
//   fp32: MFMA 32x32x2, lanes read single floats of the pixel-major tiles (channel = lane).
//   16-bit: MFMA 32x32x16, operands come from the transposing LDS read (ds_read_b64_tr_b16), whose per-lane row
//   addresses make the tap shift a plain change of address.
//   Two LDS stages; the global loads of the next sub-tile are issued before the MFMAs of the current one, parked
//   in registers and written to the other stage afterwards: one barrier per sub-tile.
#include "bn_fold.h"
#include "dev_common.h"
#include "kernels.h"

namespace oseq {

static constexpr int g_w9_wide_min = 4;  // compile-time constant: fewest sub-tiles per block for 128-channel blocks

namespace {

typedef __attribute__((ext_vector_type(16))) float v16f;
typedef __attribute__((ext_vector_type(8))) __bf16 v8bf;
typedef __attribute__((ext_vector_type(8))) _Float16 v8h;
typedef __attribute__((ext_vector_type(4))) short v4s;
typedef __attribute__((ext_vector_type(8))) short v8s;

struct W9Args {
  int N, H, W, C, K, P, Q, pad;
  int TI, TR, TC, SR, SC, NPOS, TP;  // sub-tile: images, rows, columns; staged rows / columns; positions; pixels
  int tiles_r, tiles_c, NT;          // sub-tiles per image rows / columns; in total
  int tiles_per_split;
  int xcd_group, splits;  // xcd_group: the tiles of a pixel range share an XCD (see the kernel); splits: pixel ranges
  const float* fold;  // FOLD: x is the z of a BatchNorm + ReLU, this its [4][C] statistics tensor; the staged pieces of x
                      // become the activation (scale, shift, ReLU, one rounding); positions outside the image stay zero
};

template <class T> struct W9Cfg;
template <> struct W9Cfg<float> { static constexpr int CAP = 64, MAXPOS = 144; };
template <> struct W9Cfg<bf16_t> { static constexpr int CAP = 128, MAXPOS = 256; };
template <> struct W9Cfg<f16_t> { static constexpr int CAP = 128, MAXPOS = 256; };

// WGM wavefront rows of 32 * MI output channels each (2 wavefront columns of 32 input channels): 64 * WGM threads
template <class T, int MI, int WGM> struct W9Lds {
  static constexpr bool F32 = sizeof(T) == 4;
  static constexpr int CAP = W9Cfg<T>::CAP, MAXPOS = W9Cfg<T>::MAXPOS;
  static constexpr int BMK = 32 * MI * WGM;
  static constexpr int PX = F32 ? 64 : 80;          // elements per staged x position (16-bit: 32 bytes of padding)
  static constexpr int PK = F32 ? BMK : BMK + 16;   // elements per staged dz pixel
  static constexpr int XS = MAXPOS * PX, DS = CAP * PK, STAGE = XS + DS;
  static constexpr size_t bytes = (size_t)2 * STAGE * sizeof(T) + CAP * sizeof(int);
};

__device__ __forceinline__ v16f mfma16(v8bf a, v8bf b, v16f c) { return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0); }
__device__ __forceinline__ v16f mfma16(v8h a, v8h b, v16f c) { return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0); }
template <class T> struct V8;
template <> struct V8<bf16_t> { typedef v8bf type; };
template <> struct V8<f16_t> { typedef v8h type; };
template <> struct V8<float> { typedef v8h type; };  // unused

// Two transposing 64-bit LDS reads (ds_read_b64_tr_b16).  Within a group of 16 lanes every lane supplies the address
// of 4 consecutive 16-bit elements, and lane l receives element l%4 of the addresses supplied by lanes l/4, l/4 + 4,
// l/4 + 8, l/4 + 12.  With lane r addressing channels [4*(r%4), +4) of row r/4 (of four rows), lane l therefore ends
// up with channel l of the 16 at those four rows.  p0 / p1 address the first / second group of four rows, so the
// result holds 8 consecutive reduction elements (pixels) of one channel: an MFMA operand.
template <class T>
__device__ __forceinline__ typename V8<T>::type tr_read8(const T* p0, const T* p1) {
  const v4s a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) v4s*)(p0));
  const v4s b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) v4s*)(p1));
  const v8s r = {a[0], a[1], a[2], a[3], b[0], b[1], b[2], b[3]};
  return __builtin_bit_cast(typename V8<T>::type, r);
}

// WHOLE: every sub-tile is TI whole images (small images: 8 x 8, 4 x 4).  The (row, column) part of a chunk's address and
// of its bounds check is then the same for every sub-tile: a chunk keeps its pixel index within the sub-tile, the
// sub-tile adds its first image's, and one full-rate 24-bit multiply by the channel count gives the address (pixel
// indices and channel counts are below 2^24 where this kernel is chosen) -- the general path decodes image, row and
// column, checks each against the image and multiplies them back together with quarter-rate 32- and 64-bit multiplies,
// per chunk and sub-tile, in a kernel whose instruction stream is what bounds it.
template <class T, int MI, int WGM, bool FOLD = false, bool WHOLE = false>
__global__ void __launch_bounds__(128 * WGM) __attribute__((amdgpu_waves_per_eu(WGM / 2, WGM / 2)))
conv_wgrad3x3_kernel(const T* __restrict__ x, const T* __restrict__ dz, float* __restrict__ out, W9Args a) {
  typedef W9Lds<T, MI, WGM> L;
  constexpr bool F32 = L::F32;
  constexpr int NTH = 128 * WGM;                          // threads
  constexpr int CAP = L::CAP, MAXPOS = L::MAXPOS, BMK = L::BMK, PX = L::PX, PK = L::PK;
  constexpr int EV = 16 / (int)sizeof(T);
  constexpr int XCP = 64 / EV, DCP = BMK / EV;            // 16-byte chunks per x position / dz pixel
  constexpr int XSLOTS = (MAXPOS * XCP + NTH - 1) / NTH;  // chunks per thread and sub-tile
  constexpr int DSLOTS = CAP * DCP / NTH;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  T* lds = reinterpret_cast<T*>(smem_raw);
  int* apos = reinterpret_cast<int*>(lds + 2 * L::STAGE);

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1, hg = lane >> 5, l32 = lane & 31;
  // Block coordinates: (output-channel tile, input-channel tile, pixel range).  The tiles of one pixel range all read
  // the same pixels of x and dz; workgroups go to the 8 XCDs round-robin by their linear index and every XCD has an L2
  // of its own, so with xcd_group the tiles of a range are renumbered onto one XCD, which then fetches those pixels
  // from HBM once (256 -> 256 channels at 262 144 pixels, bf16: 788 MB per launch without it for 268 MB of operands).
  // The grid's z extent is then the number of ranges rounded up to a multiple of 8.
  int bx = blockIdx.x, by = blockIdx.y, bz = blockIdx.z;
  if (a.xcd_group) {
    const unsigned tiles = gridDim.x * gridDim.y;
    const unsigned lin = blockIdx.x + gridDim.x * (blockIdx.y + gridDim.y * blockIdx.z);
    const unsigned xcd = lin & 7u, slot = lin >> 3;
    const unsigned tile = slot % tiles;
    bz = (int)((slot / tiles) * 8u + xcd);
    bx = (int)(tile % gridDim.x); by = (int)(tile / gridDim.x);
    if (bz >= a.splits) return;
  }
  const int k0 = bx * BMK, c0 = by * 64;
  const int N = a.N, H = a.H, W = a.W, C = a.C, K = a.K, P = a.P, Q = a.Q, pad = a.pad;
  const int TI = a.TI, TR = a.TR, TC = a.TC, SC = a.SC, NPOS = a.NPOS, TP = a.TP;
  const int t0 = bz * a.tiles_per_split;
  const int t1 = t0 + a.tiles_per_split < a.NT ? t0 + a.tiles_per_split : a.NT;
  const int nst = t1 > t0 ? t1 - t0 : 0;

  // position of tap (0,0) in the staged x tile for every pixel of a sub-tile (the same for all sub-tiles)
  for (int m = tid; m < CAP; m += NTH) {
    int ap = 0;
    if (m < TP) {
      const int ti = m / (TR * TC), rr = m - ti * (TR * TC);
      const int tr = rr / TC, tc = rr - tr * TC;
      ap = (ti * a.SR + tr) * SC + tc;
    }
    apos[m] = ap;
  }

  // sub-tile-independent part of this thread's chunks: (image, row, column) within the sub-tile, packed
  int xinfo[XSLOTS], dinfo[DSLOTS];
#pragma unroll
  for (int sl = 0; sl < XSLOTS; ++sl) {
    const int idx = sl * NTH + tid, pos = idx / XCP;
    int info = -1;
    if (pos < NPOS) {
      const int ti = pos / (a.SR * SC), rr = pos - ti * (a.SR * SC);
      const int sy = rr / SC, sx = rr - sy * SC;
      info = (ti << 20) | (sy << 10) | sx;
      if (WHOLE) {  // image in the high bits, (ti * H + y) * W + x in the low ones; a halo position outside the image: none
        const int y = sy - pad, xx = sx - pad;
        info = y >= 0 && y < H && xx >= 0 && xx < W ? (ti << 20) | ((ti * H + y) * W + xx) : -1;
      }
    }
    xinfo[sl] = info;
  }
#pragma unroll
  for (int sl = 0; sl < DSLOTS; ++sl) {
    const int idx = sl * NTH + tid, m = idx / DCP;
    int info = -1;
    if (m < TP) {
      const int ti = m / (TR * TC), rr = m - ti * (TR * TC);
      const int tr = rr / TC, tc = rr - tr * TC;
      info = (ti << 20) | (tr << 10) | tc;
      if (WHOLE) info = (ti << 20) | ((ti * P + tr) * Q + tc);
    }
    dinfo[sl] = info;
  }

  // Loads are unconditional (clamped to the tensor start when outside) and zeroed when written to LDS.
  Chunk xr[XSLOTS], dr[DSLOTS];
  unsigned xok = 0u, dok = 0u;
  auto gload = [&](int tile) {
    if constexpr (WHOLE) {
      const int nb = tile * TI;
      const uint32_t xbase = (uint32_t)nb * (uint32_t)(H * W), dbase = (uint32_t)nb * (uint32_t)(P * Q);
      unsigned xm = 0u, dm = 0u;
#pragma unroll
      for (int sl = 0; sl < XSLOTS; ++sl) {
        const int info = xinfo[sl];
        const bool ok = info >= 0 && nb + (info >> 20) < N;
        const uint64_t off = ok ? (uint64_t)((xbase + (uint32_t)(info & 0xfffff)) & 0xffffffu) * (uint64_t)((uint32_t)C & 0xffffffu) : 0;
        const int v = (sl * NTH + tid) % XCP;
        xr[sl] = *reinterpret_cast<const Chunk*>(x + off + c0 + v * EV);
        xm |= ok ? (1u << sl) : 0u;
      }
#pragma unroll
      for (int sl = 0; sl < DSLOTS; ++sl) {
        const int info = dinfo[sl];
        const bool ok = info >= 0 && nb + (info >> 20) < N;
        const uint64_t off = ok ? (uint64_t)((dbase + (uint32_t)(info & 0xfffff)) & 0xffffffu) * (uint64_t)((uint32_t)K & 0xffffffu) : 0;
        const int v = (sl * NTH + tid) % DCP;
        dr[sl] = *reinterpret_cast<const Chunk*>(dz + off + k0 + v * EV);
        dm |= ok ? (1u << sl) : 0u;
      }
      xok = xm; dok = dm;
      return;
    }
    const int ci = tile % a.tiles_c, t2 = tile / a.tiles_c;
    const int ri = t2 % a.tiles_r, ii = t2 / a.tiles_r;
    const int nb = ii * TI, yb = ri * TR, xb = ci * TC;
    unsigned xm = 0u, dm = 0u;
#pragma unroll
    for (int sl = 0; sl < XSLOTS; ++sl) {
      const int info = xinfo[sl];
      const int n = nb + (info >> 20), y = yb - pad + ((info >> 10) & 1023), xx = xb - pad + (info & 1023);
      const bool ok = info >= 0 && n < N && y >= 0 && y < H && xx >= 0 && xx < W;
      const int v = (sl * NTH + tid) % XCP;
      const int64_t off = ok ? (((int64_t)n * H + y) * W + xx) * C : 0;
      xr[sl] = *reinterpret_cast<const Chunk*>(x + off + c0 + v * EV);
      xm |= ok ? (1u << sl) : 0u;
    }
#pragma unroll
    for (int sl = 0; sl < DSLOTS; ++sl) {
      const int info = dinfo[sl];
      const int n = nb + (info >> 20), p = yb + ((info >> 10) & 1023), q = xb + (info & 1023);
      const bool ok = info >= 0 && n < N && p < P && q < Q;
      const int v = (sl * NTH + tid) % DCP;
      const int64_t off = ok ? (((int64_t)n * P + p) * Q + q) * K : 0;
      dr[sl] = *reinterpret_cast<const Chunk*>(dz + off + k0 + v * EV);
      dm |= ok ? (1u << sl) : 0u;
    }
    xok = xm; dok = dm;
  };
  // FOLD: a thread's pieces of x all cover the same EV channels, whose scale and shift it keeps in registers
  static_assert(NTH % XCP == 0, "a thread's pieces of x must share their channels");
  float fsc[EV], fsh[EV];
  if (FOLD) {
    load_f32<float, EV>(a.fold + 2 * C + c0 + (tid % XCP) * EV, fsc);
    load_f32<float, EV>(a.fold + 3 * C + c0 + (tid % XCP) * EV, fsh);
  }
  auto sstore = [&](int stage) {
    T* xs = lds + stage * L::STAGE;
    T* ds = xs + L::XS;
    if (FOLD) {
#pragma unroll
      for (int sl = 0; sl < XSLOTS; ++sl) xr[sl] = bn_fold_chunk<T>(xr[sl], fsc, fsh);
    }
#pragma unroll
    for (int sl = 0; sl < XSLOTS; ++sl) {
      const int idx = sl * NTH + tid, pos = idx / XCP, v = idx - pos * XCP;
      if (pos < MAXPOS) *reinterpret_cast<Chunk*>(&xs[pos * PX + v * EV]) = ((xok >> sl) & 1u) ? xr[sl] : zero_chunk();
    }
#pragma unroll
    for (int sl = 0; sl < DSLOTS; ++sl) {
      const int idx = sl * NTH + tid, m = idx / DCP, v = idx - m * DCP;
      *reinterpret_cast<Chunk*>(&ds[m * PK + v * EV]) = ((dok >> sl) & 1u) ? dr[sl] : zero_chunk();
    }
  };

  v16f acc[MI][9];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int t = 0; t < 9; ++t)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][t][e] = 0.f;

  int toff[9];  // element offset of tap t relative to tap (0,0) in the staged x tile
#pragma unroll
  for (int t = 0; t < 9; ++t) toff[t] = ((t / 3) * SC + (t % 3)) * PX;

  auto compute = [&](int stage) {
    const T* xs = lds + stage * L::STAGE;
    const T* ds = xs + L::XS;
    if constexpr (F32) {
      const float* fx = reinterpret_cast<const float*>(xs) + wn * 32 + l32;
      const float* fd = reinterpret_cast<const float*>(ds) + wm * 32 * MI + l32;
      const int nss = (TP + 7) >> 3;  // rows past the sub-tile's pixels are zero: skipped
#pragma unroll 1
      for (int ss = 0; ss < nss; ++ss) {
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          const int m = ss * 8 + hg * 4 + t;
          const float* bx = fx + apos[m] * PX;
          float av[MI];
#pragma unroll
          for (int i = 0; i < MI; ++i) av[i] = fd[m * PK + i * 32];
#pragma unroll
          for (int tap = 0; tap < 9; ++tap) {
            const float bv = bx[toff[tap]];
#pragma unroll
            for (int i = 0; i < MI; ++i) acc[i][tap] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[i], bv, acc[i][tap], 0, 0, 0);
          }
        }
      }
    } else {
      const int r16 = l32 & 15;
      const int colsel = (l32 & 16) + 4 * (r16 & 3);
      const T* tx = xs + wn * 32 + colsel;
      const T* td = ds + wm * 32 * MI + colsel;
      const int nss = (TP + 15) >> 4;
#pragma unroll 2
      for (int ss = 0; ss < nss; ++ss) {
        const int ma = ss * 16 + hg * 8 + (r16 >> 2), mb = ma + 4;
        const T* xa = tx + apos[ma] * PX;
        const T* xb = tx + apos[mb] * PX;
        typename V8<T>::type fa[MI];
#pragma unroll
        for (int i = 0; i < MI; ++i) fa[i] = tr_read8(td + ma * PK + i * 32, td + mb * PK + i * 32);
#pragma unroll
        for (int tap = 0; tap < 9; ++tap) {
          const typename V8<T>::type fb = tr_read8(xa + toff[tap], xb + toff[tap]);
#pragma unroll
          for (int i = 0; i < MI; ++i) acc[i][tap] = mfma16(fa[i], fb, acc[i][tap]);
        }
      }
    }
  };

  if (nst > 0) { gload(t0); sstore(0); }
  __syncthreads();
  for (int g = 0; g + 1 < nst; ++g) {  // steady state without range checks
    gload(t0 + g + 1);
    compute(g & 1);
    sstore((g + 1) & 1);
    __syncthreads();
  }
  if (nst > 0) compute((nst - 1) & 1);

  const int64_t outputs = (int64_t)K * 9 * C;
  float* dst = out + (int64_t)bz * outputs;
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int tap = 0; tap < 9; ++tap) {
      const int c = c0 + wn * 32 + l32;
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int k = k0 + wm * 32 * MI + i * 32 + 8 * (e >> 2) + 4 * hg + (e & 3);
        dst[((int64_t)k * 9 + tap) * C + c] = acc[i][tap][e];
      }
    }
}

// sub-tile geometry for a (P x Q) output grid: up to `cap` pixels and `maxpos` staged positions
bool w9_geometry(int N, int P, int Q, int cap, int maxpos, W9Args& a) {
  int tc = Q < cap ? Q : cap;
  int tr = cap / tc; if (tr > P) tr = P; if (tr < 1) tr = 1;
  int ti = (tr == P && tc == Q) ? cap / (P * Q) : 1;
  if (ti > N) ti = N; if (ti < 1) ti = 1;
  while (ti > 1 && ti * (tr + 2) * (tc + 2) > maxpos) ti /= 2;
  while (tr > 1 && ti * (tr + 2) * (tc + 2) > maxpos) --tr;
  while (tc > 1 && ti * (tr + 2) * (tc + 2) > maxpos) tc /= 2;
  if (ti * (tr + 2) * (tc + 2) > maxpos) return false;
  a.TI = ti; a.TR = tr; a.TC = tc; a.SR = tr + 2; a.SC = tc + 2;
  a.NPOS = ti * a.SR * a.SC; a.TP = ti * tr * tc;
  a.tiles_r = (P + tr - 1) / tr; a.tiles_c = (Q + tc - 1) / tc;
  a.NT = ((N + ti - 1) / ti) * a.tiles_r * a.tiles_c;
  return true;
}

// everything decided from the layer shape: block shape, sub-tile geometry, number of pixel ranges
struct W9Plan { W9Args a; int mi, splits; };
bool w9_plan(int dt, const ConvGeom& g, W9Plan& pl) {
  if (g.R != 3 || g.S != 3 || g.stride != 1 || g.C % 64 != 0 || g.K % 64 != 0) return false;
  if (g.H >= 1024 || g.W >= 1024) return false;  // packed (image within the sub-tile, row, column) fields
  const int cap = dt == DT_F32 ? W9Cfg<float>::CAP : W9Cfg<bf16_t>::CAP;
  const int maxpos = dt == DT_F32 ? W9Cfg<float>::MAXPOS : W9Cfg<bf16_t>::MAXPOS;
  W9Args a{};
  if (!w9_geometry(g.N, g.P, g.Q, cap, maxpos, a)) return false;
  if (a.TP * 2 < cap) return false;  // short sub-tiles: too little work between barriers
  a.N = g.N; a.H = g.H; a.W = g.W; a.C = g.C; a.K = g.K; a.P = g.P; a.Q = g.Q; a.pad = g.pad;
  // fp32: 64 output channels per block.  16-bit: 128 when possible (fewer operand fetches per MFMA), unless the blocks
  // would then get fewer than g_w9_wide_min sub-tiles each: a block's accumulators (9 taps x 64*MI x 64 floats) are
  // written out once per pixel range and read again by the reduction, and with few sub-tiles per range that traffic
  // outweighs the operand reuse (128->128 at 16x16, batch 256, bf16: 49.6 us with 64-channel blocks, 48.1 with
  // 128-channel blocks of four sub-tiles each).  At that size the 75 MB of partial sums written and read back are most
  // of the time: 19 GFLOP would take 8 us at the matrix cores' peak.
  for (int mi = (dt != DT_F32 && g.K % 128 == 0) ? 2 : 1; mi >= 1; --mi) {
    const int64_t tiles = (int64_t)(g.K / (64 * mi)) * (g.C / 64);
    int64_t s = tiles >= 256 ? 1 : (256 + tiles / 2) / tiles;  // about one block per CU
    if (s > a.NT) s = a.NT;
    if (s > 256) s = 256;
    if (s < 1) s = 1;
    a.tiles_per_split = (int)((a.NT + s - 1) / s);
    s = (a.NT + a.tiles_per_split - 1) / a.tiles_per_split;  // no empty ranges
    if (mi == 2 && a.tiles_per_split < g_w9_wide_min) continue;
    if (tiles * s < 128) return false;  // too few blocks for the chip: one tap per block does better
    pl.a = a; pl.mi = mi; pl.splits = (int)s;
    return true;
  }
  return false;
}

template <class T, int MI, int WGM, bool FOLD>
void launch_w9(hipStream_t st, const void* x, const void* dz, float* dst, const W9Plan& pl) {
  constexpr size_t sm = W9Lds<T, MI, WGM>::bytes;
  static bool attr_done = false;
  if (!attr_done) {
    (void)hipFuncSetAttribute((const void*)conv_wgrad3x3_kernel<T, MI, WGM, FOLD, false>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)sm);
    (void)hipFuncSetAttribute((const void*)conv_wgrad3x3_kernel<T, MI, WGM, FOLD, true>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)sm);
    attr_done = true;
  }
  W9Args a = pl.a;
  const int tiles = (a.K / (32 * MI * WGM)) * (a.C / 64);
  a.splits = pl.splits;
  a.xcd_group = tiles > 1 && pl.splits >= 8;  // (from the shape only)
  dim3 grid(a.K / (32 * MI * WGM), a.C / 64, a.xcd_group ? (pl.splits + 7) / 8 * 8 : pl.splits), block(128 * WGM);
  // sub-tiles of whole images, every index that is multiplied below 2^24, the pixel index within a sub-tile below 2^20
  const bool whole = a.tiles_r == 1 && a.tiles_c == 1 && a.TR == a.P && a.TC == a.Q && a.H == a.P && a.W == a.Q &&
                     (int64_t)a.N * a.H * a.W + (int64_t)a.TI * a.H * a.W < (1 << 24) && a.C < (1 << 24) && a.K < (1 << 24) &&
                     a.TI < 256 && (int64_t)a.TI * a.H * a.W < (1 << 20);
  if (whole) OSEQ_LAUNCH((conv_wgrad3x3_kernel<T, MI, WGM, FOLD, true>), grid, block, sm, st, (const T*)x, (const T*)dz, dst, a);
  else OSEQ_LAUNCH((conv_wgrad3x3_kernel<T, MI, WGM, FOLD, false>), grid, block, sm, st, (const T*)x, (const T*)dz, dst, a);
}

template <class T>
void launch_w9_16(hipStream_t st, const void* x, const void* dz, float* dst, const W9Plan& pl) {
  // 128 output channels per block: four wavefront rows of 32 channels (eight wavefronts, two per SIMD)
  if (pl.a.fold) {
    if (pl.mi == 2) launch_w9<T, 1, 4, true>(st, x, dz, dst, pl); else launch_w9<T, 1, 2, true>(st, x, dz, dst, pl);
  } else {
    if (pl.mi == 2) launch_w9<T, 1, 4, false>(st, x, dz, dst, pl); else launch_w9<T, 1, 2, false>(st, x, dz, dst, pl);
  }
}

}  // namespace

static constexpr int g_wgrad3x3 = 1;  // compile-time switch

bool conv_wgrad3x3_ok(int dt, const ConvGeom& g) {
  W9Plan pl;
  return g_wgrad3x3 && w9_plan(dt, g, pl);
}

int conv_wgrad3x3_splits(int dt, const ConvGeom& g) {
  W9Plan pl;
  return w9_plan(dt, g, pl) ? pl.splits : 1;
}

// dst: [splits][K][9][C] floats (dw itself when splits == 1); fold: see W9Args (16-bit modes only)
void launch_conv_wgrad3x3(hipStream_t st, int dt, const void* x, const void* dz, float* dst, const ConvGeom& g,
                          const float* fold) {
  W9Plan pl;
  if (!w9_plan(dt, g, pl)) return;
  pl.a.fold = dt == DT_F32 ? nullptr : fold;
  if (dt == DT_F32) launch_w9<float, 1, 2, false>(st, x, dz, dst, pl);
  else if (dt == DT_BF16) launch_w9_16<bf16_t>(st, x, dz, dst, pl);
  else launch_w9_16<f16_t>(st, x, dz, dst, pl);
}

}  // namespace oseq
