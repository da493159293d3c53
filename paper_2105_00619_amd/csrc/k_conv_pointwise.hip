// 1x1 convolutions in 16-bit storage as a plain GEMM on the matrix cores (gfx950):
//   out[m][n] = sum_c X[row(m)][c] * W[n][c]      m = output pixel, n = output channel, c = input channel
// The rows of X are whole pixels of the NHWC source (row(m) = m for stride 1; for a strided forward convolution the
// pixel (2p, 2q) of the same image), W is the (C_out, C_in) weight matrix for forward and its (C_in, C_out) transpose
// for the data gradient (of a stride-2 layer on an even image: the rows are the pixels of dz, each written to pixel
// (2p, 2q) of dx, and the three other pixels of that 2x2 cell, which no filter tap reaches, are written as zero).
// Four kernels: conv1x1_kernel (below), conv1x1_large_kernel (256 x 256 tiles for layers with many pixels),
// conv1x1_ws_kernel and conv1x1_rows_kernel (forward and data gradient of the short-depth wide layers).  These layers
// move far more bytes per flop than the 3x3 ones (depth 64 to 2048 only), so conv1x1_kernel is built to keep HBM busy
// rather than the matrix cores:
//   * block = 256 threads = 4 wavefronts (2 x 2), tile 128 rows x BN channels (BN = 128 or 64), depth step 64 bytes;
//     40 KB of LDS and at most 168 registers per lane, so three blocks share a CU and cover each other's load
//     latency, barriers and epilogue;
//   * global loads run two depth steps ahead in registers, LDS is double buffered, one barrier per step;
//   * the column tiles of one row tile get consecutive slots of the same XCD (workgroups go to the 8 XCDs round-robin
//     by index), so the X tile is fetched from HBM once and re-read from that XCD's L2;
//   * epilogue through LDS: bias / residual addend / ReLU in fp32, one rounding, 16-byte stores of whole rows, and the
//     per-block channel sums of the stored values for the BatchNorm that follows.
#include "bn_fold.h"
#include "dev_common.h"
#include "epilogue.h"
#include "kernels.h"

namespace oseq {
namespace {

typedef __attribute__((ext_vector_type(16))) float v16f;
typedef __attribute__((ext_vector_type(8))) __bf16 v8bf;
typedef __attribute__((ext_vector_type(8))) _Float16 v8h;
typedef __attribute__((ext_vector_type(4))) float v4f;

template <class T> struct Mma;
template <> struct Mma<bf16_t> {
  typedef v8bf V;
  __device__ static __forceinline__ v16f run(V a, V b, v16f c) { return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0); }
};
template <> struct Mma<f16_t> {
  typedef v8h V;
  __device__ static __forceinline__ v16f run(V a, V b, v16f c) { return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0); }
};

struct PwArgs {
  int64_t M;              // output pixels
  int Ng, Kd;             // output channels, depth (input channels)
  int MT, NT;             // row tiles, column tiles
  int relu;
  int stride;             // 1, or 2: row m = (n, p, q) reads source pixel (n, 2p, 2q)
  int scatter;            // data gradient of a stride-2 layer: row m = (n, p, q) is written to pixel (n, 2p, 2q) of a
                          // (2 dstH) x (2 dstW) image and its three neighbours get zero (plus the addend)
  int dstH, dstW, srcH, srcW;
  FastDiv div_w, div_hw;  // by dstW and dstH * dstW
  const uint8_t* amask;   // data gradient with an addend: ReLU bit mask the addend is multiplied by, or null
  const float* fold;      // forward: X is the z of a BatchNorm + ReLU whose [4][Kd] statistics tensor this is; the rows are
                          //          turned into the activation (scale, shift, ReLU, one rounding) on their way to LDS
};

template <int V> struct IC { static constexpr int value = V; };

constexpr int PW_BM = 128;
constexpr int PW_BK = 32;              // elements per depth step (64 bytes)
constexpr int PW_PITCH = PW_BK + 8;    // LDS row pitch in elements (80 bytes)

template <int BN> constexpr size_t pw_smem_bytes() {
  constexpr size_t stages = (size_t)2 * (PW_BM + BN) * PW_PITCH * 2;
  constexpr size_t epi = (size_t)(PW_BM / 2) * (BN + 4) * 4;
  return stages > epi ? stages : epi;
}

// Data gradient of a stride-2 layer: block row r (pixel (n, p, q) of dz) goes to pixel (n, 2p, 2q) of dx, and the three
// other pixels of that 2x2 cell get zero; with an addend every one of the four adds its own addend values (all loads
// of a row before its stores).
template <class T, int BN>
__device__ __forceinline__ void scatter_rows(const float* ep, int tid, int n0, int64_t mbase, const T* __restrict__ addend,
                                             T* __restrict__ out, const PwArgs& a) {
  constexpr int EP_PITCH = BN + 4;
  constexpr int GROUPS = BN / 8;
  constexpr int PER_THREAD = 64 * GROUPS / 256;
  constexpr int RG = 256 / GROUPS;
  const int c8 = (tid % GROUPS) * 8, erow = tid / GROUPS;
  const int col = n0 + c8;
  const int fullW = 2 * a.dstW;
#pragma unroll
  for (int it = 0; it < PER_THREAD; ++it) {
    const int row = erow + it * RG;
    const int64_t grow = mbase + row;
    if (grow >= a.M) continue;
    const uint32_t mm = (uint32_t)grow;
    const uint32_t n = a.div_hw.div(mm), rem = mm - n * a.div_hw.d;
    const uint32_t p = a.div_w.div(rem), q = rem - p * a.div_w.d;
    const int64_t o00 = ((int64_t)n * (2 * a.dstH) + 2 * p) * fullW + 2 * q;
    const v4f x0 = *reinterpret_cast<const v4f*>(&ep[row * EP_PITCH + c8]);
    const v4f x1 = *reinterpret_cast<const v4f*>(&ep[row * EP_PITCH + c8 + 4]);
    float w8[4][8];
#pragma unroll
    for (int k = 0; k < 8; ++k) { w8[0][k] = k < 4 ? x0[k] : x1[k - 4]; w8[1][k] = 0.f; w8[2][k] = 0.f; w8[3][k] = 0.f; }
    if (addend) {
      Vec<T, 8> ad[4];
#pragma unroll
      for (int sib = 0; sib < 4; ++sib)
        ad[sib] = *reinterpret_cast<const Vec<T, 8>*>(addend + (o00 + (sib >> 1) * fullW + (sib & 1)) * a.Ng + col);
#pragma unroll
      for (int sib = 0; sib < 4; ++sib)
#pragma unroll
        for (int k = 0; k < 8; ++k) w8[sib][k] += to_f32(ad[sib].v[k]);
    }
#pragma unroll
    for (int sib = 0; sib < 4; ++sib) store_f32<T, 8>(out + (o00 + (sib >> 1) * fullW + (sib & 1)) * a.Ng + col, w8[sib]);
  }
}

// DGRAD: the data-gradient instantiation (addend and scatter, no bias / ReLU / sums); else the forward one
// (FOLD needs some forty registers more: two blocks per CU instead of three)
template <class T, int BN, bool DGRAD, bool FOLD = false>
__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(FOLD ? 2 : 3, FOLD ? 2 : 3)))
conv1x1_kernel(const T* __restrict__ X, const T* __restrict__ W, const float* __restrict__ bias, const T* __restrict__ addend,
               T* __restrict__ out, float* __restrict__ stat_partial, PwArgs a) {
  typedef typename Mma<T>::V FV;
  constexpr int BM = PW_BM, BK = PW_BK, PITCH = PW_PITCH;
  constexpr int MI = 2, NI = BN / 64;      // 32x32 MFMA tiles per wavefront
  constexpr int A_CH = BM * 4 / 256;       // 16-byte chunks per thread and depth step
  constexpr int B_CH = BN * 4 / 256;
  constexpr int STAGE = (BM + BN) * PITCH;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  T* lds = reinterpret_cast<T*>(smem_raw);

  // slot s of XCD x: column tile s % NT of row tile (s / NT) * 8 + x
  const int b = blockIdx.x, xcd = b & 7, slot = b >> 3;
  const int nt = slot % a.NT, mt = (slot / a.NT) * 8 + xcd;
  if (mt >= a.MT) return;
  const int64_t m0 = (int64_t)mt * BM;
  const int n0 = nt * BN;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1, g = lane >> 5, l32 = lane & 31;
  const int vec = tid & 3, row0 = tid >> 2;
  const int Kd = a.Kd;

  // Rows past the last pixel read row 0; their sums are never stored.
  const T* arow[A_CH];
#pragma unroll
  for (int i = 0; i < A_CH; ++i) {
    const int64_t m = m0 + row0 + i * 64;
    int64_t r = m < a.M ? m : 0;
    if (a.stride != 1) {
      const uint32_t mm = (uint32_t)r;
      const uint32_t n = a.div_hw.div(mm), rem = mm - n * a.div_hw.d;
      const uint32_t p = a.div_w.div(rem), q = rem - p * a.div_w.d;
      r = ((int64_t)n * a.srcH + p * a.stride) * a.srcW + q * a.stride;
    }
    arow[i] = X + r * Kd + vec * 8;
  }
  const T* brow[B_CH];
#pragma unroll
  for (int i = 0; i < B_CH; ++i) brow[i] = W + (int64_t)(n0 + row0 + i * 64) * Kd + vec * 8;

  Chunk ra[2][A_CH], rb[2][B_CH];
  auto gload = [&](auto P, int kt) {
    constexpr int p = decltype(P)::value;
#pragma unroll
    for (int i = 0; i < A_CH; ++i) ra[p][i] = *reinterpret_cast<const Chunk*>(arow[i] + kt * BK);
#pragma unroll
    for (int i = 0; i < B_CH; ++i) rb[p][i] = *reinterpret_cast<const Chunk*>(brow[i] + kt * BK);
  };
  // FOLD: scale and shift of all Kd channels lie in LDS behind the stages; the pieces of tile kt become activations
  float* ftab = reinterpret_cast<float*>(smem_raw + pw_smem_bytes<BN>());  // [2][Kd]
  if (FOLD) {
    for (int i = tid; i < Kd; i += 256) { ftab[i] = a.fold[2 * Kd + i]; ftab[Kd + i] = a.fold[3 * Kd + i]; }
    __syncthreads();
  }
  auto sstore = [&](auto P, int stage, int kt) {
    constexpr int p = decltype(P)::value;
    T* st = lds + stage * STAGE;
    if (FOLD) {
      float sc[8], sh[8];
      load_f32<float, 8>(ftab + kt * BK + vec * 8, sc);
      load_f32<float, 8>(ftab + Kd + kt * BK + vec * 8, sh);
#pragma unroll
      for (int i = 0; i < A_CH; ++i) ra[p][i] = bn_fold_chunk<T>(ra[p][i], sc, sh);
    }
#pragma unroll
    for (int i = 0; i < A_CH; ++i) *reinterpret_cast<Chunk*>(&st[(row0 + i * 64) * PITCH + vec * 8]) = ra[p][i];
#pragma unroll
    for (int i = 0; i < B_CH; ++i) *reinterpret_cast<Chunk*>(&st[(BM + row0 + i * 64) * PITCH + vec * 8]) = rb[p][i];
  };

  v16f acc[MI][NI];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NI; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  // lane group g owns depth elements [16g, 16g + 16) of a step; A and B pair the same indices, so the sum is the same
  const int afrag = (wm * 64 + l32) * PITCH + g * 16;
  const int bfrag = (BM + wn * (BN / 2) + l32) * PITCH + g * 16;
  auto compute = [&](int stage) {
    const T* st = lds + stage * STAGE;
    FV fa[MI][2], fb[NI][2];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
#pragma unroll
      for (int i = 0; i < MI; ++i) fa[i][h] = *reinterpret_cast<const FV*>(st + afrag + i * 32 * PITCH + h * 8);
#pragma unroll
      for (int j = 0; j < NI; ++j) fb[j][h] = *reinterpret_cast<const FV*>(st + bfrag + j * 32 * PITCH + h * 8);
    }
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
      for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j) acc[i][j] = Mma<T>::run(fa[i][h], fb[j][h], acc[i][j]);
  };

  // Step j: the registers of generation j & 1 (tile j) go to LDS stage j & 1 and are refilled with tile j + 2; one
  // barrier, then the MFMAs of tile j.  A stage is rewritten two steps later, after the barrier of the step between,
  // which every wavefront passes only when it is done reading.  The steady loop is unconditional straight-line code;
  // the last two steps (no refill) are peeled.
  const int n = Kd / BK;  // >= 2
  gload(IC<0>{}, 0);
  gload(IC<1>{}, 1);
  int j = 0;
  for (; j + 3 < n; j += 2) {
    sstore(IC<0>{}, 0, j); gload(IC<0>{}, j + 2); __syncthreads(); compute(0);
    sstore(IC<1>{}, 1, j + 1); gload(IC<1>{}, j + 3); __syncthreads(); compute(1);
  }
  if (j + 2 < n) {  // odd number of steps: three left
    sstore(IC<0>{}, 0, j); gload(IC<0>{}, j + 2); __syncthreads(); compute(0);
    sstore(IC<1>{}, 1, j + 1); __syncthreads(); compute(1);
    sstore(IC<0>{}, 0, j + 2); __syncthreads(); compute(0);
  } else {
    sstore(IC<0>{}, 0, j); __syncthreads(); compute(0);
    sstore(IC<1>{}, 1, j + 1); __syncthreads(); compute(1);
  }

  // ---- epilogue: the rows of one wavefront pair at a time through LDS as fp32 [64][BN + 4]; the store half (bias /
  // addend / ReLU, rounding, stores of whole rows, BatchNorm sums) is shared with the other kernels ----------------
  float* ep = reinterpret_cast<float*>(smem_raw);
  constexpr int EP_PITCH = BN + 4;
  float ss[8], qq[8];
#pragma unroll
  for (int k = 0; k < 8; ++k) { ss[k] = 0.f; qq[k] = 0.f; }
#pragma unroll
  for (int u = 0; u < 2; ++u) {
    __syncthreads();
    if (wm == u) {
#pragma unroll
      for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int jn = 0; jn < NI; ++jn)
#pragma unroll
          for (int e = 0; e < 16; ++e)
            ep[(i * 32 + 8 * (e >> 2) + 4 * g + (e & 3)) * EP_PITCH + wn * (BN / 2) + jn * 32 + l32] = acc[i][jn][e];
    }
    __syncthreads();
    auto rowoff = [&](int row) -> int64_t {
      const int64_t grow = m0 + u * 64 + row;
      return grow < a.M ? grow * a.Ng : -1;
    };
    if (DGRAD) {
      if (a.scatter) scatter_rows<T, BN>(ep, tid, n0, m0 + u * 64, addend, out, a);
      else epi_store_pass<T, BN, 64, false, true, false>(ep, tid, n0, bias, addend, a.amask, out, 0, rowoff, ss, qq);
    } else {
      if (stat_partial) epi_store_pass<T, BN, 64, true, false, true>(ep, tid, n0, bias, addend, nullptr, out, a.relu, rowoff, ss, qq);
      else epi_store_pass<T, BN, 64, true, false, false>(ep, tid, n0, bias, addend, nullptr, out, a.relu, rowoff, ss, qq);
    }
  }
  if (!DGRAD && stat_partial)
    epi_stat_combine<BN>(ep, tid, ss, qq, stat_partial + ((int64_t)mt * 2 + 0) * a.Ng + n0,
                         stat_partial + ((int64_t)mt * 2 + 1) * a.Ng + n0);
}

// The same GEMM with a 256 x 256 tile for layers with many pixels (stride 1, no scatter).  Operand tiles travel from L2
// to the CUs at about 10 TB/s over the whole chip, and a block of this kernel family moves (BM + BN) * depth elements
// for BM * BN results: with 128 x 128 tiles a layer of the bottleneck networks at batch 4096 moves 2.1 GB that way and
// cannot finish faster than ~210 us, whatever HBM and the matrix cores could do; 256 x 256 tiles halve that.  512
// threads = 8 wavefronts (2 x 4), wave tile 128 x 64 (MI = 4, NI = 2: six operand reads from LDS per eight MFMAs instead of
// four per four), 80 KB of LDS: one block per CU, two wavefronts per SIMD.  A layer with 256 output channels reads its
// activations exactly once.  The column tiles of a row tile again take consecutive slots of one XCD.  Measured at
// 262 144 pixels, bf16: 1024 -> 256 channels 222 -> 184 us, its data gradient 213 -> 170 us, 256 -> 1024 channels
// 300 -> 265 us; tiles of 128 x 256 and 256 x 128 with two blocks per CU lie between (195-202 us on the first).
constexpr int PWL_BM = 256, PWL_BN = 256;

template <int BM, int BN> constexpr size_t pwl_smem_bytes() {
  constexpr size_t stages = (size_t)2 * (BM + BN) * PW_PITCH * 2;
  constexpr size_t epi = (size_t)64 * (BN + 4) * 4;
  return stages > epi ? stages : epi;
}

// BM x BN tile, WGM x WGN wavefronts (wave tile BM / WGM x BN / WGN, at least 64 rows)
template <class T, bool DGRAD, int BM, int BN, int WGM, int WGN, bool FOLD = false>
__global__ void __launch_bounds__(64 * WGM * WGN) __attribute__((amdgpu_waves_per_eu(2, 2)))
conv1x1_large_kernel(const T* __restrict__ X, const T* __restrict__ W, const float* __restrict__ bias,
                     const T* __restrict__ addend, T* __restrict__ out, float* __restrict__ stat_partial, PwArgs a) {
  typedef typename Mma<T>::V FV;
  constexpr int NT = 64 * WGM * WGN, BK = PW_BK, PITCH = PW_PITCH;
  constexpr int WTM = BM / WGM, WTN = BN / WGN;       // wave tile
  constexpr int MI = WTM / 32, NI = WTN / 32;
  static_assert(WTM >= 64 && WTM % 64 == 0, "the epilogue moves 64 rows of one wavefront row at a time");
  constexpr int A_CH = BM * 4 / NT;        // 16-byte chunks per thread and depth step
  constexpr int B_CH = BN * 4 / NT;
  constexpr int RSTEP = NT / 4;            // rows between a thread's chunks
  constexpr int STAGE = (BM + BN) * PITCH;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  T* lds = reinterpret_cast<T*>(smem_raw);

  // slot s of XCD x: column tile s % NT of row tile (s / NT) * 8 + x
  const int b = blockIdx.x, xcd = b & 7, slot = b >> 3;
  const int nt = slot % a.NT, mt = (slot / a.NT) * 8 + xcd;
  if (mt >= a.MT) return;
  const int64_t m0 = (int64_t)mt * BM;
  const int n0 = nt * BN;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WGN, wn = wave % WGN, g = lane >> 5, l32 = lane & 31;
  const int vec = tid & 3, row0 = tid >> 2;
  const int Kd = a.Kd;

  // Rows past the last pixel read row 0; they are never stored and add nothing to the sums.
  const T* arow[A_CH];
#pragma unroll
  for (int i = 0; i < A_CH; ++i) {
    const int64_t m = m0 + row0 + i * RSTEP;
    arow[i] = X + (m < a.M ? m : 0) * Kd + vec * 8;
  }
  const T* brow[B_CH];
#pragma unroll
  for (int i = 0; i < B_CH; ++i) brow[i] = W + (int64_t)(n0 + row0 + i * RSTEP) * Kd + vec * 8;

  Chunk ra[2][A_CH], rb[2][B_CH];
  auto gload = [&](auto P, int kt) {
    constexpr int p = decltype(P)::value;
#pragma unroll
    for (int i = 0; i < A_CH; ++i) ra[p][i] = *reinterpret_cast<const Chunk*>(arow[i] + kt * BK);
#pragma unroll
    for (int i = 0; i < B_CH; ++i) rb[p][i] = *reinterpret_cast<const Chunk*>(brow[i] + kt * BK);
  };
  float* ftab = reinterpret_cast<float*>(smem_raw + pwl_smem_bytes<BM, BN>());  // FOLD: [2][Kd] scale, shift
  if (FOLD) {
    for (int i = tid; i < Kd; i += NT) { ftab[i] = a.fold[2 * Kd + i]; ftab[Kd + i] = a.fold[3 * Kd + i]; }
    __syncthreads();
  }
  auto sstore = [&](auto P, int stage, int kt) {
    constexpr int p = decltype(P)::value;
    T* st = lds + stage * STAGE;
    if (FOLD) {
      float sc[8], sh[8];
      load_f32<float, 8>(ftab + kt * BK + vec * 8, sc);
      load_f32<float, 8>(ftab + Kd + kt * BK + vec * 8, sh);
#pragma unroll
      for (int i = 0; i < A_CH; ++i) ra[p][i] = bn_fold_chunk<T>(ra[p][i], sc, sh);
    }
#pragma unroll
    for (int i = 0; i < A_CH; ++i) *reinterpret_cast<Chunk*>(&st[(row0 + i * RSTEP) * PITCH + vec * 8]) = ra[p][i];
#pragma unroll
    for (int i = 0; i < B_CH; ++i) *reinterpret_cast<Chunk*>(&st[(BM + row0 + i * RSTEP) * PITCH + vec * 8]) = rb[p][i];
  };

  v16f acc[MI][NI];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NI; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  const int afrag = (wm * WTM + l32) * PITCH + g * 16;
  const int bfrag = (BM + wn * WTN + l32) * PITCH + g * 16;
  auto compute = [&](int stage) {
    const T* st = lds + stage * STAGE;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      FV fa[MI], fb[NI];
#pragma unroll
      for (int i = 0; i < MI; ++i) fa[i] = *reinterpret_cast<const FV*>(st + afrag + i * 32 * PITCH + h * 8);
#pragma unroll
      for (int j = 0; j < NI; ++j) fb[j] = *reinterpret_cast<const FV*>(st + bfrag + j * 32 * PITCH + h * 8);
#pragma unroll
      for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j) acc[i][j] = Mma<T>::run(fa[i], fb[j], acc[i][j]);
    }
  };

  // The two-generation pipeline of conv1x1_kernel as one uniform loop (an even number of depth steps): the last two
  // refills load the last tile again (the same addresses, just read) and are never used -- peeled steps without the
  // loads cost this kernel, which holds 128 accumulator registers, a few hundred spilled registers per thread.  (Four
  // tiles in flight instead of two changed nothing: 187 against 184 us on 1024 -> 256 channels at 262 144 pixels.)
  const int n = Kd / BK;  // even, >= 2
  gload(IC<0>{}, 0);
  gload(IC<1>{}, 1);
  for (int j = 0; j < n; j += 2) {
    const int t2 = j + 2 < n ? j + 2 : n - 1, t3 = j + 3 < n ? j + 3 : n - 1;
    sstore(IC<0>{}, 0, j); gload(IC<0>{}, t2); __syncthreads(); compute(0);
    sstore(IC<1>{}, 1, j + 1); gload(IC<1>{}, t3); __syncthreads(); compute(1);
  }

  // ---- epilogue: 64 rows at a time through LDS as fp32 [64][BN + 4] (the rows of the four wavefronts with wm = pass / 2,
  // their 32-row tiles 2 * (pass & 1) and + 1), stored by all 512 threads ------------------------------------------------
  float* ep = reinterpret_cast<float*>(smem_raw);
  constexpr int EP_PITCH = BN + 4;
  float ss[8], qq[8];
#pragma unroll
  for (int k = 0; k < 8; ++k) { ss[k] = 0.f; qq[k] = 0.f; }
  // a data gradient that adds a residual: the addend pieces of pass p + 1 are requested before the stores of pass p
  constexpr int EPT = 64 * (BN / 8) / NT;
  Vec<T, 8> adn[EPT];
  unsigned mbn[EPT];
  const bool residual = DGRAD && addend != nullptr;
  auto rowoff_of = [&](int pass) {
    return [&a, m0, pass](int row) -> int64_t {
      const int64_t grow = m0 + pass * 64 + row;
      return grow < a.M ? grow * a.Ng : -1;
    };
  };
  if (residual) epi_load_addend_nt<NT, T, BN, 64>(tid, n0, addend, a.amask, rowoff_of(0), adn, mbn);
#pragma unroll
  for (int pass = 0; pass < BM / 64; ++pass) {
    __syncthreads();
    if (wm == pass * 64 / WTM) {
#pragma unroll
      for (int ii = 0; ii < 2; ++ii)
#pragma unroll
        for (int jn = 0; jn < NI; ++jn)
#pragma unroll
          for (int e = 0; e < 16; ++e)
            ep[(ii * 32 + 8 * (e >> 2) + 4 * g + (e & 3)) * EP_PITCH + wn * WTN + jn * 32 + l32] =
                acc[(pass * 64 % WTM) / 32 + ii][jn][e];
    }
    __syncthreads();
    auto rowoff = rowoff_of(pass);
    if (residual) {
      Vec<T, 8> ad[EPT];
      unsigned mb[EPT];
#pragma unroll
      for (int it = 0; it < EPT; ++it) { ad[it] = adn[it]; mb[it] = mbn[it]; }
      if (pass + 1 < BM / 64) epi_load_addend_nt<NT, T, BN, 64>(tid, n0, addend, a.amask, rowoff_of(pass + 1), adn, mbn);
      epi_store_rows_pre_nt<NT, T, BN, 64>(ep, tid, n0, ad, mb, out, rowoff);
    } else if (DGRAD) {
      epi_store_pass_nt<NT, T, BN, 64, false, true, false>(ep, tid, n0, bias, addend, a.amask, out, 0, rowoff, ss, qq);
    } else {
      if (stat_partial) epi_store_pass_nt<NT, T, BN, 64, true, false, true>(ep, tid, n0, bias, addend, nullptr, out, a.relu, rowoff, ss, qq);
      else epi_store_pass_nt<NT, T, BN, 64, true, false, false>(ep, tid, n0, bias, addend, nullptr, out, a.relu, rowoff, ss, qq);
    }
  }
  if (!DGRAD && stat_partial)
    epi_stat_combine_nt<NT, BN>(ep, tid, ss, qq, stat_partial + ((int64_t)mt * 2 + 0) * a.Ng + n0,
                                stat_partial + ((int64_t)mt * 2 + 1) * a.Ng + n0);
}

// Short-depth, wide layers (depth 64 to 256, two to four times as many output channels: the last convolution of a
// bottleneck block and the data gradient of its first).  A tile of the kernels above spends a few depth steps between a start-up that
// waits for HBM and an epilogue that stores 128 KB, and most of its instructions in that epilogue; and it fetches the
// weight matrix from L2 again for every row tile, more bytes than HBM moves for these layers.  Two kernels for them:
//
// Data gradient (conv1x1_rows_kernel): a block keeps its 128 rows of dz, all of their depth, resident in LDS and walks
// the column tiles (256 channels each) itself: dz is read from HBM exactly once and from L2 never; the weight tiles
// stream through two LDS stages of 128 bytes of depth from registers two steps ahead, the stream running on across
// the column tiles, so that the loads of the next tile's first steps (and the next residual pieces) are in flight
// while this tile's results are stored.  512 threads = 8 wavefronts (2 x 4), wave tile 64 x 64.  Epilogue of a column
// tile with a residual: 64 rows at a time through LDS as fp32, the masked residual added before the rounding; without
// one: rounded on the accumulators where they are, the rounded values through LDS as [128][256 + 8] elements; 16-byte
// stores of whole rows either way.
constexpr int PWR_BM = 128, PWR_BN = 256, PWR_BK = 64;
constexpr int PWR_PITCH = PWR_BK + 8;  // LDS row pitch of a weight stage in elements (144 bytes)

template <int KD> constexpr size_t pwr_smem_bytes() {
  return (size_t)2 * PWR_BN * PWR_PITCH * 2 + (size_t)PWR_BM * (KD + 8) * 2;
}

template <class T, int KD>
__global__ void __launch_bounds__(512)
conv1x1_rows_kernel(const T* __restrict__ X, const T* __restrict__ W, const T* __restrict__ addend, T* __restrict__ out,
                    PwArgs a) {
  typedef typename Mma<T>::V FV;
  constexpr int NT = 512, BM = PWR_BM, BN = PWR_BN, BK = PWR_BK, PITCH = PWR_PITCH, APITCH = KD + 8;
  constexpr int WGN = 4, MI = 2, NI = 2;
  constexpr int NS = KD / BK;          // depth steps per column tile (2 or 4)
  constexpr int CPR = KD / 8;          // 16-byte chunks per row of X
  constexpr int A_CH = BM * CPR / NT;  // of them per thread
  constexpr int RPI = NT / CPR;        // rows between a thread's chunks
  constexpr int B_CH = BN * (BK / 8) / NT;  // chunks per thread of a weight stage (4)
  constexpr int BSTAGE = BN * PITCH;
  constexpr int HR = 64;               // rows per pass of the residual-adding epilogue (a wavefront row)
  constexpr int EPITCH = BN + 8;       // row pitch of the rounded tile
  static_assert(NS == 2 || NS == 4, "depth 128 or 256");
  static_assert((size_t)BM * EPITCH * 2 <= (size_t)2 * BSTAGE * 2, "the rounded tile lies over the weight stages");
  static_assert((size_t)HR * (BN + 4) * 4 <= (size_t)2 * BSTAGE * 2, "so does the fp32 tile of the residual-adding epilogue");
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  T* bst = reinterpret_cast<T*>(smem_raw);
  T* ares = bst + 2 * BSTAGE;
  float* ep = reinterpret_cast<float*>(smem_raw);
  T* stg = reinterpret_cast<T*>(smem_raw);

  const int mt = blockIdx.x;
  const int64_t m0 = (int64_t)mt * BM;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WGN, wn = wave % WGN, g = lane >> 5, l32 = lane & 31;
  const int vec = tid & 7, row0 = tid >> 3;  // a weight stage: 8 chunks per row, 64 rows per sweep of the block
  const int NP = a.Ng / BN, last = NP * NS - 1;

  // weight stream: step t = depth step t % NS of column tile t / NS
  const T* bbase = W + (int64_t)row0 * KD + vec * 8;
  Chunk rb[2][B_CH];
  auto gload = [&](auto P, int t) {
    constexpr int p = decltype(P)::value;
    const T* src = bbase + (int64_t)(t / NS) * BN * KD + (t % NS) * BK;
#pragma unroll
    for (int i = 0; i < B_CH; ++i) rb[p][i] = *reinterpret_cast<const Chunk*>(src + (int64_t)i * 64 * KD);
  };
  auto sstore = [&](auto P) {
    constexpr int p = decltype(P)::value;
    T* st = bst + p * BSTAGE;
#pragma unroll
    for (int i = 0; i < B_CH; ++i) *reinterpret_cast<Chunk*>(&st[(row0 + i * 64) * PITCH + vec * 8]) = rb[p][i];
  };
  gload(IC<0>{}, 0);
  gload(IC<1>{}, 1);

  // the block's rows of X, whole depth; rows past the last pixel read row 0 (never stored)
  {
    const int cc = tid % CPR, r0 = tid / CPR;
    Chunk ra[A_CH];
#pragma unroll
    for (int i = 0; i < A_CH; ++i) {
      const int64_t m = m0 + r0 + i * RPI;
      ra[i] = *reinterpret_cast<const Chunk*>(X + (m < a.M ? m : 0) * KD + cc * 8);
    }
#pragma unroll
    for (int i = 0; i < A_CH; ++i) *reinterpret_cast<Chunk*>(&ares[(r0 + i * RPI) * APITCH + cc * 8]) = ra[i];
  }

  v16f acc[MI][NI];
  // lane group g owns depth elements [32 s + 16 g, + 16) of the two 32-element halves s of a step, 8 per MFMA
  const int afrag = (wm * 64 + l32) * APITCH + g * 16;
  const int bfrag = (wn * 64 + l32) * PITCH + g * 16;
  auto compute = [&](int stage, int kt) {
    const T* st = bst + stage * BSTAGE;
    const T* ar = ares + kt * BK;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int ko = (q >> 1) * 32 + (q & 1) * 8;
      FV fa[MI], fb[NI];
#pragma unroll
      for (int i = 0; i < MI; ++i) fa[i] = *reinterpret_cast<const FV*>(ar + afrag + i * 32 * APITCH + ko);
#pragma unroll
      for (int j = 0; j < NI; ++j) fb[j] = *reinterpret_cast<const FV*>(st + bfrag + j * 32 * PITCH + ko);
#pragma unroll
      for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j) acc[i][j] = Mma<T>::run(fa[i], fb[j], acc[i][j]);
    }
  };

  constexpr int EPT = HR * (BN / 8) / NT;
  Vec<T, 8> adn[EPT];
  unsigned mbn[EPT];
  const bool residual = addend != nullptr;
  auto rowoff_of = [&](int sp) {
    return [&a, m0, sp](int row) -> int64_t {
      const int64_t grow = m0 + sp * HR + row;
      return grow < a.M ? grow * a.Ng : -1;
    };
  };
  if (residual) epi_load_addend_nt<NT, T, BN, HR>(tid, 0, addend, a.amask, rowoff_of(0), adn, mbn);
  const bool ragged = m0 + BM > a.M;

  for (int ps = 0; ps < NP; ++ps) {
    const int n0 = ps * BN;
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
      for (int j = 0; j < NI; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
    // A step stores its generation to LDS and refills it with the step two ahead (past the end: the last step again,
    // never used); a stage is rewritten two steps later, after the barrier of the step between.
#pragma unroll
    for (int k2 = 0; k2 < NS; k2 += 2) {
      const int t = ps * NS + k2;
      sstore(IC<0>{}); gload(IC<0>{}, t + 2 < last ? t + 2 : last); __syncthreads(); compute(0, k2);
      sstore(IC<1>{}); gload(IC<1>{}, t + 3 < last ? t + 3 : last); __syncthreads(); compute(1, k2 + 1);
    }
    __syncthreads();  // the weight stages are free: the epilogue tiles lie over them

    if (residual) {
      // ---- 64 rows at a time as fp32 [64][BN + 4]; the residual pieces of a pass are requested a pass ahead ----
#pragma unroll
      for (int sp = 0; sp < BM / HR; ++sp) {
        if (sp) __syncthreads();
        if (wm == sp) {
#pragma unroll
          for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int jn = 0; jn < NI; ++jn)
#pragma unroll
              for (int e = 0; e < 16; ++e)
                ep[(i * 32 + 8 * (e >> 2) + 4 * g + (e & 3)) * (BN + 4) + wn * 64 + jn * 32 + l32] = acc[i][jn][e];
        }
        __syncthreads();
        Vec<T, 8> ad[EPT];
        unsigned mb[EPT];
#pragma unroll
        for (int it = 0; it < EPT; ++it) { ad[it] = adn[it]; mb[it] = mbn[it]; }
        if (sp + 1 < BM / HR) epi_load_addend_nt<NT, T, BN, HR>(tid, n0, addend, a.amask, rowoff_of(sp + 1), adn, mbn);
        else if (ps + 1 < NP) epi_load_addend_nt<NT, T, BN, HR>(tid, n0 + BN, addend, a.amask, rowoff_of(0), adn, mbn);
        epi_store_rows_pre_nt<NT, T, BN, HR>(ep, tid, n0, ad, mb, out, rowoff_of(sp));
      }
    } else {
      // ---- rounded in place (a lane holds pairs of consecutive rows of one channel), through LDS as [BM][EPITCH] ----
#pragma unroll
      for (int jn = 0; jn < NI; ++jn) {
        const int cj = wn * 64 + jn * 32 + l32;
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
          for (int e = 0; e < 16; e += 2) {  // rows r and r + 1: one packed conversion
            const int r = wm * 64 + i * 32 + 8 * (e >> 2) + 4 * g + (e & 3);
            const typename Pair16<T>::V q = from_f32x2<T>(acc[i][jn][e], acc[i][jn][e + 1]);
            stg[r * EPITCH + cj] = q[0];
            stg[(r + 1) * EPITCH + cj] = q[1];
          }
      }
      __syncthreads();
      constexpr int SPT = BM * (BN / 8) / NT;  // 16-byte pieces per thread
      const int c8 = (tid % (BN / 8)) * 8, erow = tid / (BN / 8);
#pragma unroll
      for (int it = 0; it < SPT; ++it) {
        const int row = erow + it * (NT / (BN / 8));
        const Chunk c = *reinterpret_cast<const Chunk*>(&stg[row * EPITCH + c8]);
        if (!ragged || m0 + row < a.M) *reinterpret_cast<Chunk*>(out + (m0 + row) * a.Ng + n0 + c8) = c;
      }
    }
    __syncthreads();  // the weight stages are free again
  }
}

// Forward (conv1x1_ws_kernel), weights stationary: a block owns 256 output channels for its whole life -- every
// wavefront keeps the weights of its 32 channels, all of their depth, in registers as MFMA operands (64 registers at
// depth 256) -- and walks row tiles of 128 (depth 256: 64) pixels: a tile of X goes through LDS once (turned into
// activations on the way if a BatchNorm is folded in) and is multiplied by all eight wavefronts (wave tile 128 x 32,
// or 64 x 32).
// Per tile nothing but X crosses from L2 to the CU.  256 blocks, one per CU; the blocks that share row tiles (one per
// 256 channels) take consecutive slots of one XCD and move through the tiles together.  The next tile of X is requested
// before the MFMAs of the current one and waits in registers.  Epilogue: bias / ReLU / rounding on the accumulators
// where they are (a lane holds pairs of consecutive rows of one channel: the BatchNorm sums of the rounded values are
// two dot-product instructions per pair, kept in registers over all tiles, one row of block sums per block), the
// rounded values through LDS, 16-byte stores of whole rows.
constexpr int PWS_BN = 256, PWS_BLOCKS = 256;
// rows per tile: at depth 256 the weights take 64 registers, and 128 rows (64 accumulator registers, 32 for the tile in
// flight) no longer fit beside them
constexpr int pws_bm(int kd) { return kd > 128 ? 64 : 128; }

template <int KD> constexpr size_t pws_smem_bytes() {
  return (size_t)pws_bm(KD) * (KD + 8) * 2 + (size_t)pws_bm(KD) * (PWS_BN + 8) * 2 + (size_t)2 * 2 * PWS_BN * 4 + (size_t)2 * KD * 4;
}

template <class T, bool FOLD, int KD>
__global__ void __launch_bounds__(512)
conv1x1_ws_kernel(const T* __restrict__ X, const T* __restrict__ W, const float* __restrict__ bias, T* __restrict__ out,
                  float* __restrict__ stat_partial, PwArgs a) {
  typedef typename Mma<T>::V FV;
  typedef typename Dot2<T>::V T2;
  constexpr int NT = 512, BM = pws_bm(KD), BN = PWS_BN, APITCH = KD + 8, EPITCH = BN + 8;
  constexpr int MI = BM / 32, KC = KD / 16;  // 32-row tiles per wavefront, 16-deep MFMA steps
  constexpr int CPR = KD / 8;          // 16-byte chunks per row of X
  constexpr int A_CH = BM * CPR / NT;  // of them per thread
  constexpr int RPI = NT / CPR;        // rows between a thread's chunks
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  T* abuf = reinterpret_cast<T*>(smem_raw);           // [BM][APITCH]: the tile of X
  T* stg = abuf + BM * APITCH;                        // [BM][EPITCH]: the rounded results
  float* red = reinterpret_cast<float*>(stg + BM * EPITCH);  // [2][2][BN]
  float* ftab = red + 2 * 2 * BN;                     // FOLD: [2][KD] scale, shift

  // slot s of XCD x: channel group s % NCG of row group (s / NCG) * 8 + x
  const int NCG = a.Ng / BN, RGN = PWS_BLOCKS / NCG;
  const int b = blockIdx.x, xcd = b & 7, slot = b >> 3;
  const int cg = slot % NCG, rg = (slot / NCG) * 8 + xcd;
  const int n0 = cg * BN;
  const int MT = a.MT;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int g = lane >> 5, l32 = lane & 31;
  const int cj = wave * 32 + l32;  // the lane's channel within the block's 256

  // the lane's weights: lane group g owns depth elements [32 s + 16 g, + 16) of every 32, 8 per MFMA
  FV fb[KC];
  {
    const T* wrow = W + (int64_t)(n0 + cj) * KD + g * 16;
#pragma unroll
    for (int q = 0; q < KC; ++q) fb[q] = *reinterpret_cast<const FV*>(wrow + (q >> 1) * 32 + (q & 1) * 8);
  }
  if (FOLD) {
    for (int i = tid; i < KD; i += NT) { ftab[i] = a.fold[2 * KD + i]; ftab[KD + i] = a.fold[3 * KD + i]; }
  }
  const float bj = bias ? bias[n0 + cj] : 0.f;

  const int cc = tid % CPR, r0 = tid / CPR;
  Chunk ra[A_CH];
  // A tile's loads: one base for the block plus offsets that are the same for every tile; only the last tile can have
  // rows past the last pixel, which read row 0 (never stored, nothing added to the sums)
  const int xoff = r0 * KD + cc * 8;
  auto gload = [&](int t) {
    const int64_t m0t = (int64_t)t * BM;
    if (m0t + BM <= a.M) {
      const T* Xt = X + m0t * KD;
#pragma unroll
      for (int i = 0; i < A_CH; ++i) ra[i] = *reinterpret_cast<const Chunk*>(Xt + (xoff + i * (RPI * KD)));
    } else {
#pragma unroll
      for (int i = 0; i < A_CH; ++i) {
        const int64_t m = m0t + r0 + i * RPI;
        ra[i] = *reinterpret_cast<const Chunk*>(X + (m < a.M ? m : 0) * KD + cc * 8);
      }
    }
  };
  const int afrag = l32 * APITCH + g * 16;
  const int c8 = (tid % (BN / 8)) * 8, erow = tid / (BN / 8);
  float S1 = 0.f, S2 = 0.f;
  T2 one2;
  one2[0] = from_f32<T>(1.f); one2[1] = from_f32<T>(1.f);

  // `ra` -> LDS (as activations if a BatchNorm is folded in), then the request for the tile after it
  auto stage_tile = [&](int tnext) {
    if (FOLD) {
      float sc[8], sh[8];
      load_f32<float, 8>(ftab + cc * 8, sc);
      load_f32<float, 8>(ftab + KD + cc * 8, sh);
#pragma unroll
      for (int i = 0; i < A_CH; ++i) ra[i] = bn_fold_chunk<T>(ra[i], sc, sh);
    }
#pragma unroll
    for (int i = 0; i < A_CH; ++i) *reinterpret_cast<Chunk*>(&abuf[(r0 + i * RPI) * APITCH + cc * 8]) = ra[i];
    if (tnext < MT) gload(tnext);
  };

  // Two barriers per row tile: the MFMAs of tile t and the rounding of its results into `stg` between them; then the
  // stores of tile t from `stg` together with the staging of tile t + 1 into `abuf`.  Loads and stores share one
  // in-order counter: the rows a tile waits for were requested before the stores of the tile before it.
  int t = rg;  // < MT
  gload(t);
  if (FOLD) __syncthreads();  // the scale / shift table
  stage_tile(t + RGN);
  for (;;) {
    __syncthreads();
    v16f acc[MI];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;
#pragma unroll
    for (int q = 0; q < KC; ++q) {
      FV fa[MI];
#pragma unroll
      for (int i = 0; i < MI; ++i)
        fa[i] = *reinterpret_cast<const FV*>(abuf + afrag + i * 32 * APITCH + (q >> 1) * 32 + (q & 1) * 8);
#pragma unroll
      for (int i = 0; i < MI; ++i) acc[i] = Mma<T>::run(fa[i], fb[q], acc[i]);
    }

    const int64_t m0 = (int64_t)t * BM;
    const bool ragged = m0 + BM > a.M;
    // whether the tile has rows past the last pixel is the same for the whole block: one branch per tile picks the
    // straight-line variant, instead of compares and selects per element
    auto round_tile = [&](auto GENERAL, auto RAGGED) {
      constexpr bool rag = decltype(RAGGED)::value != 0, general = decltype(GENERAL)::value != 0;
      const bool relu = general && a.relu != 0;
      float s1 = 0.f, s2 = 0.f;
#pragma unroll
      for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int e = 0; e < 16; e += 2) {
          const int r = i * 32 + 8 * (e >> 2) + 4 * g + (e & 3);  // and r + 1
          float v0 = acc[i][e], v1 = acc[i][e + 1];
          if (general) { v0 += bj; v1 += bj; }
          if (relu) { v0 = fmaxf(v0, 0.f); v1 = fmaxf(v1, 0.f); }
          if (rag) {  // rows past the last pixel count as zero
            if (m0 + r >= a.M) v0 = 0.f;
            if (m0 + r + 1 >= a.M) v1 = 0.f;
          }
          const T2 p2 = from_f32x2<T>(v0, v1);
          s1 = Dot2<T>::run(p2, one2, s1);
          s2 = Dot2<T>::run(p2, p2, s2);
          stg[r * EPITCH + cj] = p2[0];
          stg[(r + 1) * EPITCH + cj] = p2[1];
        }
      S1 += s1; S2 += s2;
    };
    // a convolution in front of a BatchNorm has neither bias nor ReLU: its tiles (but a ragged last one) take the
    // version without either
    if (ragged) round_tile(IC<1>{}, IC<1>{});
    else if (bias || a.relu) round_tile(IC<1>{}, IC<0>{});
    else round_tile(IC<0>{}, IC<0>{});
    __syncthreads();
    {
      T* ot = out + m0 * a.Ng + n0;  // the tile's first row at the block's first channel: the same for every thread
      const int ooff = erow * a.Ng + c8, ostep = (NT / (BN / 8)) * a.Ng;
#pragma unroll
      for (int it = 0; it < BM * (BN / 8) / NT; ++it) {
        const int row = erow + it * (NT / (BN / 8));
        const Chunk c = *reinterpret_cast<const Chunk*>(&stg[row * EPITCH + c8]);
        if (!ragged || m0 + row < a.M) *reinterpret_cast<Chunk*>(ot + (ooff + it * ostep)) = c;
      }
    }
    t += RGN;
    if (t >= MT) break;
    stage_tile(t + RGN);
  }
  if (stat_partial) {  // the two lane groups of a channel in a fixed order
    red[g * BN + cj] = S1;
    red[(2 + g) * BN + cj] = S2;
    __syncthreads();
    if (tid < BN) {
      stat_partial[((int64_t)rg * 2 + 0) * a.Ng + n0 + tid] = red[tid] + red[BN + tid];
      stat_partial[((int64_t)rg * 2 + 1) * a.Ng + n0 + tid] = red[2 * BN + tid] + red[3 * BN + tid];
    }
  }
}

template <class T, bool FOLD, int KD>
void launch_pw_ws(hipStream_t st, const void* X, const void* W, const float* bias, void* out, float* stat_partial, PwArgs a) {
  constexpr size_t sm = pws_smem_bytes<KD>();
  static bool attr_done = false;
  if (!attr_done) {
    (void)hipFuncSetAttribute((const void*)conv1x1_ws_kernel<T, FOLD, KD>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)sm);
    attr_done = true;
  }
  a.MT = ceil_div(a.M, pws_bm(KD));
  a.NT = a.Ng / PWS_BN;
  OSEQ_LAUNCH((conv1x1_ws_kernel<T, FOLD, KD>), dim3(PWS_BLOCKS), dim3(512), sm, st, (const T*)X, (const T*)W, bias, (T*)out,
              stat_partial, a);
}

// from the shape only: depth 64, 128 or 256 and at least twice as many output channels; 1, 2, 4 ... 32 channel groups;
// at least four row tiles per block
bool pw_ws_ok(int64_t M, int Ng, int Kd, int stride) {
  if (stride != 1 || (Kd != 64 && Kd != 128 && Kd != 256) || Ng % PWS_BN != 0 || Ng < 2 * Kd) return false;
  const int ncg = Ng / PWS_BN;
  if (ncg > 32 || (ncg & (ncg - 1)) != 0) return false;
  return ceil_div(M, 128) >= 4 * (PWS_BLOCKS / ncg);
}

template <class T, int KD>
void launch_pw_ws_t(hipStream_t st, const void* X, const void* W, const float* bias, void* out, float* stat_partial, const PwArgs& a) {
  if (a.fold) launch_pw_ws<T, true, KD>(st, X, W, bias, out, stat_partial, a);
  else launch_pw_ws<T, false, KD>(st, X, W, bias, out, stat_partial, a);
}

template <class T, int KD>
void launch_pw_rows(hipStream_t st, const void* X, const void* W, const void* addend, void* out, PwArgs a) {
  constexpr size_t sm = pwr_smem_bytes<KD>();
  static bool attr_done = false;
  if (!attr_done) {
    (void)hipFuncSetAttribute((const void*)conv1x1_rows_kernel<T, KD>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)sm);
    attr_done = true;
  }
  a.MT = ceil_div(a.M, PWR_BM);
  a.NT = a.Ng / PWR_BN;
  OSEQ_LAUNCH((conv1x1_rows_kernel<T, KD>), dim3(a.MT), dim3(512), sm, st, (const T*)X, (const T*)W, (const T*)addend, (T*)out, a);
}

// from the shape only: at least two blocks per CU
bool pw_rows_ok(int64_t M, int Ng, int Kd, int stride, bool scatter) {
  if (stride != 1 || scatter || (Kd != 128 && Kd != 256) || Ng % PWR_BN != 0 || Ng < 2 * PWR_BN) return false;
  return ceil_div(M, PWR_BM) >= 512;
}

constexpr int PW_FOLD_MAX_DEPTH = 1024;  // the scale / shift table of a folded BatchNorm takes 8 bytes of LDS per channel

template <class T, bool DGRAD, int BM, int BN, int WGM, int WGN, bool FOLD>
void launch_pw_large(hipStream_t st, const void* X, const void* W, const float* bias, const void* addend, void* out,
                     float* stat_partial, PwArgs a) {
  constexpr size_t sm = pwl_smem_bytes<BM, BN>();
  static bool attr_done = false;
  if (!attr_done) {
    (void)hipFuncSetAttribute((const void*)conv1x1_large_kernel<T, DGRAD, BM, BN, WGM, WGN, FOLD>,
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)(sm + (FOLD ? PW_FOLD_MAX_DEPTH * 8 : 0)));
    attr_done = true;
  }
  a.MT = ceil_div(a.M, BM);
  a.NT = a.Ng / BN;
  const int grid = ((a.MT + 7) / 8) * 8 * a.NT;
  OSEQ_LAUNCH((conv1x1_large_kernel<T, DGRAD, BM, BN, WGM, WGN, FOLD>), dim3(grid), dim3(64 * WGM * WGN),
              sm + (FOLD ? (size_t)a.Kd * 8 : 0), st, (const T*)X, (const T*)W, bias, (const T*)addend, (T*)out, stat_partial, a);
}

// The 256 x 256 tile is taken when the layer still gives every CU two blocks of it (from the shape only).
bool pw_large_ok(int64_t M, int Ng, int Kd, int stride, bool scatter) {
  if (stride != 1 || scatter || Ng % PWL_BN != 0 || Kd % (2 * PW_BK) != 0) return false;
  return (int64_t)ceil_div(M, PWL_BM) * (Ng / PWL_BN) >= 512;
}

template <class T, int BN, bool DGRAD, bool FOLD>
void launch_pw_v(hipStream_t st, const void* X, const void* W, const float* bias, const void* addend, void* out,
                 float* stat_partial, const PwArgs& a) {
  constexpr size_t sm = pw_smem_bytes<BN>();
  static bool attr_done = false;
  if (!attr_done) {
    (void)hipFuncSetAttribute((const void*)conv1x1_kernel<T, BN, DGRAD, FOLD>, hipFuncAttributeMaxDynamicSharedMemorySize,
                              (int)(sm + (FOLD ? PW_FOLD_MAX_DEPTH * 8 : 0)));
    attr_done = true;
  }
  const int grid = ((a.MT + 7) / 8) * 8 * a.NT;
  OSEQ_LAUNCH((conv1x1_kernel<T, BN, DGRAD, FOLD>), dim3(grid), dim3(256), sm + (FOLD ? (size_t)a.Kd * 8 : 0), st,
              (const T*)X, (const T*)W, bias, (const T*)addend, (T*)out, stat_partial, a);
}

template <class T>
void launch_pw_t(hipStream_t st, bool dgrad, int bn, const void* X, const void* W, const float* bias, const void* addend,
                 void* out, float* stat_partial, const PwArgs& a) {
  if (dgrad) {
    if (bn == 128) launch_pw_v<T, 128, true, false>(st, X, W, bias, addend, out, stat_partial, a);
    else launch_pw_v<T, 64, true, false>(st, X, W, bias, addend, out, stat_partial, a);
  } else if (a.fold) {
    if (bn == 128) launch_pw_v<T, 128, false, true>(st, X, W, bias, addend, out, stat_partial, a);
    else launch_pw_v<T, 64, false, true>(st, X, W, bias, addend, out, stat_partial, a);
  } else {
    if (bn == 128) launch_pw_v<T, 128, false, false>(st, X, W, bias, addend, out, stat_partial, a);
    else launch_pw_v<T, 64, false, false>(st, X, W, bias, addend, out, stat_partial, a);
  }
}

// A data gradient that adds a residual takes 256 x 128 tiles with two blocks per CU: its block spends more time in the
// epilogue (fetching the 128 KB residual tile, storing as much) than in its depth loop, and with the CU to itself
// nothing overlaps the two (256 -> 1024 channels at 262 144 pixels, bf16: 354 us with 128 x 128 tiles, 353 with
// 256 x 256 and the residual fetched a pass ahead, 340 with 256 x 128).  The same half tile for short-depth forward
// layers was far slower (the class 47 -> 60 ms per step on the largest workload).
template <class T>
void launch_pw_large_t(hipStream_t st, bool dgrad, const void* X, const void* W, const float* bias, const void* addend,
                       void* out, float* stat_partial, const PwArgs& a) {
  if (dgrad && addend) launch_pw_large<T, true, PWL_BM, PWL_BN / 2, 2, 2, false>(st, X, W, bias, addend, out, stat_partial, a);
  else if (dgrad) launch_pw_large<T, true, PWL_BM, PWL_BN, 2, 4, false>(st, X, W, bias, addend, out, stat_partial, a);
  else if (a.fold) launch_pw_large<T, false, PWL_BM, PWL_BN, 2, 4, true>(st, X, W, bias, addend, out, stat_partial, a);
  else launch_pw_large<T, false, PWL_BM, PWL_BN, 2, 4, false>(st, X, W, bias, addend, out, stat_partial, a);
}

void launch_pw(hipStream_t st, int dt, bool dgrad, const void* X, const void* W, const float* bias, const void* addend,
               void* out, float* stat_partial, PwArgs a) {
  if (!dgrad && pw_ws_ok(a.M, a.Ng, a.Kd, a.stride)) {
    if (dt == DT_BF16) {
      if (a.Kd == 256) launch_pw_ws_t<bf16_t, 256>(st, X, W, bias, out, stat_partial, a);
      else if (a.Kd == 128) launch_pw_ws_t<bf16_t, 128>(st, X, W, bias, out, stat_partial, a);
      else launch_pw_ws_t<bf16_t, 64>(st, X, W, bias, out, stat_partial, a);
    } else {
      if (a.Kd == 256) launch_pw_ws_t<f16_t, 256>(st, X, W, bias, out, stat_partial, a);
      else if (a.Kd == 128) launch_pw_ws_t<f16_t, 128>(st, X, W, bias, out, stat_partial, a);
      else launch_pw_ws_t<f16_t, 64>(st, X, W, bias, out, stat_partial, a);
    }
    return;
  }
  if (dgrad && pw_rows_ok(a.M, a.Ng, a.Kd, a.stride, a.scatter != 0)) {
    if (dt == DT_BF16) {
      if (a.Kd == 256) launch_pw_rows<bf16_t, 256>(st, X, W, addend, out, a);
      else launch_pw_rows<bf16_t, 128>(st, X, W, addend, out, a);
    } else {
      if (a.Kd == 256) launch_pw_rows<f16_t, 256>(st, X, W, addend, out, a);
      else launch_pw_rows<f16_t, 128>(st, X, W, addend, out, a);
    }
    return;
  }
  if (pw_large_ok(a.M, a.Ng, a.Kd, a.stride, a.scatter != 0)) {
    if (dt == DT_BF16) launch_pw_large_t<bf16_t>(st, dgrad, X, W, bias, addend, out, stat_partial, a);
    else launch_pw_large_t<f16_t>(st, dgrad, X, W, bias, addend, out, stat_partial, a);
    return;
  }
  const int bn = a.Ng % 128 == 0 ? 128 : 64;
  a.MT = ceil_div(a.M, PW_BM);
  a.NT = a.Ng / bn;
  if (dt == DT_BF16) launch_pw_t<bf16_t>(st, dgrad, bn, X, W, bias, addend, out, stat_partial, a);
  else launch_pw_t<f16_t>(st, dgrad, bn, X, W, bias, addend, out, stat_partial, a);
}

// shapes the kernel takes: 16-bit storage, depth a multiple of the step and at least two steps, and enough blocks
// (below half a block per CU the depth-split GEMM fills the chip better)
bool pw_shape_ok(int dt, int64_t M, int Ng, int Kd, int min_blocks) {
  if (dt == DT_F32 || Kd % PW_BK != 0 || Kd < 2 * PW_BK || Ng % 64 != 0) return false;
  if (M >= ((int64_t)1 << 31)) return false;
  const int64_t blocks = (int64_t)ceil_div(M, PW_BM) * (Ng / (Ng % 128 == 0 ? 128 : 64));
  return blocks >= min_blocks;
}

}  // namespace

static constexpr int g_pointwise = 1;               // compile-time switches
static constexpr int g_pointwise_min_blocks = 128;

bool conv_pointwise_fwd_ok(int dt, const ConvGeom& g) {
  if (!g_pointwise || g.R != 1 || g.S != 1 || g.pad != 0 || (g.stride != 1 && g.stride != 2)) return false;
  return pw_shape_ok(dt, (int64_t)g.N * g.P * g.Q, g.K, g.C, g_pointwise_min_blocks);
}
bool conv_pointwise_dgrad_ok(int dt, const ConvGeom& g) {
  if (!g_pointwise || g.R != 1 || g.S != 1 || g.pad != 0) return false;
  if (g.stride == 2) {  // rows = pixels of dz, each scattered to a 2x2 cell of dx
    if (g.H != 2 * g.P || g.W != 2 * g.Q || (int64_t)g.N * g.H * g.W >= ((int64_t)1 << 31)) return false;
    return pw_shape_ok(dt, (int64_t)g.N * g.P * g.Q, g.C, g.K, g_pointwise_min_blocks);
  }
  if (g.stride != 1) return false;
  return pw_shape_ok(dt, (int64_t)g.N * g.H * g.W, g.C, g.K, g_pointwise_min_blocks);
}
int conv_pointwise_stat_blocks(const ConvGeom& g) {
  const int64_t M = (int64_t)g.N * g.P * g.Q;
  if (pw_ws_ok(M, g.K, g.C, g.stride)) return PWS_BLOCKS / (g.K / PWS_BN);
  return ceil_div(M, pw_large_ok(M, g.K, g.C, g.stride, false) ? PWL_BM : PW_BM);
}

// May the forward kernel take the z of a BatchNorm as its input and apply that BatchNorm (+ReLU) itself?
bool conv_pointwise_fold_ok(int dt, const ConvGeom& g) { return conv_pointwise_fwd_ok(dt, g) && g.C <= PW_FOLD_MAX_DEPTH; }

// fold: null, or the [4][C_in] statistics tensor of the BatchNorm whose z the tensor x is (see PwArgs::fold)
void launch_conv_fwd_pointwise(hipStream_t st, int dt, const void* x, const void* w, const float* bias, void* out,
                               float* stat_partial, const ConvGeom& g, int relu, const float* fold) {
  PwArgs a{};
  a.fold = fold;
  a.M = (int64_t)g.N * g.P * g.Q; a.Ng = g.K; a.Kd = g.C; a.relu = relu; a.stride = g.stride;
  a.dstH = g.P; a.dstW = g.Q; a.srcH = g.H; a.srcW = g.W;
  a.div_w = make_fastdiv((uint32_t)g.Q); a.div_hw = make_fastdiv((uint32_t)(g.P * g.Q));
  launch_pw(st, dt, false, x, w, bias, nullptr, out, stat_partial, a);
}

// wt: the (C_in, C_out) transpose of the weights in the compute type
void launch_conv_dgrad_pointwise(hipStream_t st, int dt, const void* dz, const void* wt, const void* addend,
                                 const uint8_t* addend_mask, void* dx, const ConvGeom& g) {
  PwArgs a{};
  a.amask = addend_mask;  // (stride-1 layers only: the identity shortcut of a block)
  a.Ng = g.C; a.Kd = g.K; a.relu = 0; a.stride = 1;
  a.scatter = g.stride == 2;
  a.dstH = a.scatter ? g.P : g.H; a.dstW = a.scatter ? g.Q : g.W; a.srcH = g.P; a.srcW = g.Q;
  a.M = (int64_t)g.N * a.dstH * a.dstW;
  a.div_w = make_fastdiv((uint32_t)a.dstW); a.div_hw = make_fastdiv((uint32_t)(a.dstH * a.dstW));
  launch_pw(st, dt, true, dz, wt, nullptr, addend, dx, nullptr, a);
}

}  // namespace oseq
