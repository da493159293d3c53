// Host-callable launchers of the HIP kernels.  Plain device pointers and sizes; `dt` is the storage type of
// activations and 16-bit weight copies (0 fp32, 1 bf16, 2 fp16).  All launches are asynchronous on `st`.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace oseq {

enum { DT_F32 = 0, DT_BF16 = 1, DT_F16 = 2 };

struct ConvGeom { int N, H, W, C, K, R, S, stride, pad, P, Q; };

void launch_cast_in(hipStream_t st, int dt, const float* x, void* out, int64_t n);
// storage type -> fp32 (read-back of an activation for inspection)
void launch_cast_out(hipStream_t st, int dt, const void* x, float* out, int64_t n);
void launch_bn_stats(hipStream_t st, int dt, const void* z, int64_t rows, int C, int nblk, float* partial, float eps,
                     float mom, const float* gamma, const float* beta, float* stats, float* running, const int* flags);
// flags[1] != 0 (an invalid label in this step's batch) keeps `running` as it is.
// the same from per-block sums a convolution already produced: partial [nblk][2][C]
// (with many blocks the rows are first folded into bn_stats_fold_rows(nblk) rows, written behind the block sums:
// partial has room for [nblk + bn_stats_fold_rows(nblk)][2][C] floats)
int bn_stats_fold_rows(int nblk);
void launch_bn_stats_finalize(hipStream_t st, float* partial, int64_t rows, int C, int nblk, float eps, float mom,
                              const float* gamma, const float* beta, float* stats, float* running, const int* flags);
// inference mode: (mean, rstd, scale, shift) from the running statistics [2][C] instead of the batch
void launch_bn_eval_stats(hipStream_t st, const float* running, const float* gamma, const float* beta, float eps, int C,
                          float* stats);
// mask (null, or with a skip connection and C a multiple of 16 / element size): receives the ReLU decisions as bits,
// byte (row * C + c) / V for the V = 16 / element size channels from c
void launch_bn_apply(hipStream_t st, int dt, const void* z, const float* stats, const void* skip, void* out, void* mask,
                     int64_t rows, int C, int relu);
// BatchNorm apply and the 2x2 max-pool behind it in one pass (H, W even): z [N][H][W][C] -> a (may be null: not kept)
// and y [N][H/2][W/2][C]
void launch_bn_apply_pool(hipStream_t st, int dt, const void* z, const float* stats, void* a, void* y, int N, int H, int W,
                          int C, int relu);
// ReLU decisions: from mask (bits as launch_bn_apply writes them, applied whatever relu says) if given, else from the
// sign of aout if given, else redone from z when relu is set
void launch_bn_bwd(hipStream_t st, int dt, const void* da, const void* z, const void* aout, const void* mask,
                   const float* stats, int64_t rows, int C, int relu, int nblk, float* ws, float* dgamma, float* dbeta,
                   void* dz, void* dskip);
// the same where dy is the gradient of the 2x2 max-pool that follows the activation ([N][H/2][W/2][C]; H, W even): the
// pool's own backward pass is not run
void launch_bn_bwd_pool(hipStream_t st, int dt, const void* dy, const void* z, const float* stats, int N, int H, int W, int C,
                        int relu, int nblk, float* ws, float* dgamma, float* dbeta, void* dz);
void launch_relu_bwd(hipStream_t st, int dt, const void* da, const void* a, void* dz, int64_t rows, int C);
void launch_bias_grad(hipStream_t st, int dt, const void* dz, int64_t rows, int C, int nblk, float* partial, float* dbias);
void launch_maxpool_fwd(hipStream_t st, int dt, const void* x, void* y, int N, int H, int W, int C);
void launch_maxpool_bwd(hipStream_t st, int dt, const void* x, const void* dy, void* dx, int N, int H, int W, int C);

void launch_head_fwd(hipStream_t st, int dt, const void* x, int N, int HW, int C, int gap, int F, int J, const float* w,
                     const float* b, const int32_t* y, float gscale, float* feat, float* logits, float* dlogits,
                     float* loss_n, float* loss_out, int* flags);
// forward of the head up to the logits (no loss): inference
void launch_head_logits(hipStream_t st, int dt, const void* x, int N, int HW, int C, int gap, int F, int J, const float* w,
                        const float* b, float* feat, float* logits);
void launch_head_bwd(hipStream_t st, int dt, const float* feat, const float* dlogits, const float* w, int N, int HW, int C,
                     int gap, int F, int J, float* dw, float* db, float* dfeat, void* dx);

void launch_conv_fwd_direct(hipStream_t st, int dt, const void* x, const void* w, const float* bias, void* out,
                            const ConvGeom& g, int relu);
void launch_conv_dgrad_direct(hipStream_t st, int dt, const void* dz, const void* w, const void* addend, void* dx,
                              const ConvGeom& g);
void launch_conv_wgrad_direct(hipStream_t st, int dt, const void* x, const void* dz, float* dw, float* partial, int splits,
                              const ConvGeom& g);

// few input channels (the stem): plain-FMA kernels with the weights in LDS
bool conv_smallc_fwd_ok(const ConvGeom& g);
bool conv_smallc_wgrad_ok(const ConvGeom& g);
int conv_smallc_wgrad_splits(const ConvGeom& g);
void launch_conv_fwd_smallc(hipStream_t st, int dt, const void* x, const void* w, const float* bias, void* out,
                            const ConvGeom& g, int relu);
void launch_conv_wgrad_smallc(hipStream_t st, int dt, const void* x, const void* dz, float* dw, float* partial, int splits,
                              const ConvGeom& g);

// matrix-core implicit GEMM (k_conv_mfma.hip); the *_ok predicates depend on the layer shape only
bool conv_mfma_fwd_ok(int dt, const ConvGeom& g);
bool conv_mfma_dgrad_ok(int dt, const ConvGeom& g);
int conv_mfma_fwd_splits(int dt, const ConvGeom& g);
int conv_mfma_dgrad_splits(int dt, const ConvGeom& g);
// partial: fp32 workspace of splits * (output elements) floats when splits > 1, else unused
int conv_mfma_fwd_stat_blocks(int dt, const ConvGeom& g);
// fold (null: none): x is not the input activation but the z of the BatchNorm + ReLU in front of the layer, and fold
// that BatchNorm's [4][C_in] statistics tensor (mean, rstd, scale, shift): the kernel turns z into the activation --
// the very values the apply kernel would have stored -- while it stages its operand.  Only where conv_fold_fwd_ok /
// conv_fold_wgrad_ok say so (from the layer shape only), and only for a BatchNorm that is followed by a ReLU.
bool conv_fold_fwd_ok(int dt, const ConvGeom& g);
bool conv_fold_wgrad_ok(int dt, const ConvGeom& g);
void launch_conv_fwd_mfma(hipStream_t st, int dt, const void* x, const void* w, const float* bias, void* out,
                          float* partial, float* stat_partial, int splits, const ConvGeom& g, int relu,
                          const float* fold = nullptr);
// addend_mask (null, or with an addend): ReLU decisions as bits (as launch_bn_apply writes them); the addend counts
// as zero where its bit is clear
void launch_conv_dgrad_mfma(hipStream_t st, int dt, const void* dz, const void* wt, const void* addend,
                            const void* addend_mask, void* dx, float* partial, int splits, const ConvGeom& g);
// 1x1 convolutions in 16-bit storage as a streaming GEMM (k_conv_pointwise.hip); used by the MFMA launchers above
bool conv_pointwise_fwd_ok(int dt, const ConvGeom& g);
bool conv_pointwise_dgrad_ok(int dt, const ConvGeom& g);
int conv_pointwise_stat_blocks(const ConvGeom& g);
bool conv_pointwise_fold_ok(int dt, const ConvGeom& g);
void launch_conv_fwd_pointwise(hipStream_t st, int dt, const void* x, const void* w, const float* bias, void* out,
                               float* stat_partial, const ConvGeom& g, int relu, const float* fold);
void launch_conv_dgrad_pointwise(hipStream_t st, int dt, const void* dz, const void* wt, const void* addend,
                                 const uint8_t* addend_mask, void* dx, const ConvGeom& g);
// 3x3 stride-1 weight gradient with all nine taps per block (k_conv_wgrad3x3.hip); used by the MFMA launcher below
bool conv_wgrad3x3_ok(int dt, const ConvGeom& g);
int conv_wgrad3x3_splits(int dt, const ConvGeom& g);
void launch_conv_wgrad3x3(hipStream_t st, int dt, const void* x, const void* dz, float* dst, const ConvGeom& g,
                          const float* fold);
bool conv_mfma_wgrad_ok(int dt, const ConvGeom& g);
int conv_mfma_wgrad_splits(int dt, const ConvGeom& g);
void launch_conv_wgrad_mfma(hipStream_t st, int dt, const void* x, const void* dz, float* dw, float* partial, int splits,
                            const ConvGeom& g, const float* fold = nullptr);
// Transposed weight copies for the data-gradient GEMMs, all layers in one launch (per 48 layers).  w_off: element
// offset of the layer's weights in the flat parameter vector (the same offset is used in the transposed copy).
struct TransposeJob { int64_t w_off; int K, RS, C, first_block; };
struct TransposeBatch { static constexpr int MAX_JOBS = 48; TransposeJob job[MAX_JOBS]; int n; };
void launch_weight_transposes(hipStream_t st, int dt, const float* wbase, void* wtbase, const TransposeJob* jobs, int njobs);

// device address and size of the per-GPU static activation arena (optorch_seq_step_static), current device
hipError_t static_arena(void** ptr, uint64_t* bytes);
void launch_step_init(hipStream_t st, int* flags, const int32_t* y, int n, int classes);
void launch_optim(hipStream_t st, int dt, float* w, float* v, const float* g, void* w16, float* gout, int64_t n, float lr,
                  float mom, float inv_scale, int* flags);
void launch_cast_params(hipStream_t st, int dt, const float* w, void* w16, int64_t n);
void launch_fill(hipStream_t st, float* p, int64_t n, float v);

// Image data-flow (x uint8 [B][P]; a uint64 [ceil(B / z)][P][words]; o uint32 [ceil(B / z)][P]); z and the pointers
// are validated by the callers.  scale / shift: host arrays of `channels` (<= 16) floats.
void launch_encode(hipStream_t st, const uint8_t* x, int64_t B, int64_t P, int z, uint64_t* a);
void launch_decode(hipStream_t st, const uint64_t* a, int64_t B, int64_t P, int z, uint8_t* x);
void launch_decode_cast(hipStream_t st, int dt, const uint64_t* a, int64_t B, int64_t P, int z, int channels,
                        const float* scale, const float* shift, void* out);
void launch_encode_lossless(hipStream_t st, const uint8_t* x, int64_t B, int64_t P, int z, uint64_t* a, uint32_t* o);
void launch_decode_lossless(hipStream_t st, const uint64_t* a, const uint32_t* o, int64_t B, int64_t P, int z, uint8_t* x);

}  // namespace oseq
