// 1x1 convolutions in 16-bit storage as a plain GEMM on the matrix cores (gfx950):
//   out[m][n] = sum_c X[row(m)][c] * W[n][c]      m = output pixel, n = output channel, c = input channel
// The rows of X are whole pixels of the NHWC source (row(m) = m for stride 1; for a strided forward convolution the
// pixel (2p, 2q) of the same image), W is the (C_out, C_in) weight matrix for forward and its (C_in, C_out) transpose
// for the data gradient (of a stride-2 layer on an even image: the rows are the pixels of dz, each written to pixel
// (2p, 2q) of dx, and the three other pixels of that 2x2 cell, which no filter tap reaches, are written as zero).  These layers move far more bytes per flop than the 3x3 ones (depth 64 to
// 2048 only), so the kernel is built to keep HBM busy rather than the matrix cores:
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
  const float* fold;      // forward: X is the z of a BatchNorm whose [4][Kd] statistics tensor this is; the rows are turned
  int fold_relu;          //          into the activation (scale, shift, ReLU if fold_relu, one rounding) on their way to LDS
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
      for (int i = 0; i < A_CH; ++i) ra[p][i] = bn_fold_chunk<T>(ra[p][i], sc, sh, a.fold_relu);
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
      for (int i = 0; i < A_CH; ++i) ra[p][i] = bn_fold_chunk<T>(ra[p][i], sc, sh, a.fold_relu);
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
  return ceil_div(M, pw_large_ok(M, g.K, g.C, g.stride, false) ? PWL_BM : PW_BM);
}

// May the forward kernel take the z of a BatchNorm as its input and apply that BatchNorm (+ReLU) itself?
bool conv_pointwise_fold_ok(int dt, const ConvGeom& g) { return conv_pointwise_fwd_ok(dt, g) && g.C <= PW_FOLD_MAX_DEPTH; }

// fold: null, or the [4][C_in] statistics tensor of the BatchNorm whose z the tensor x is (see PwArgs::fold)
void launch_conv_fwd_pointwise(hipStream_t st, int dt, const void* x, const void* w, const float* bias, void* out,
                               float* stat_partial, const ConvGeom& g, int relu, const float* fold, int fold_relu) {
  PwArgs a{};
  a.fold = fold; a.fold_relu = fold_relu;
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
