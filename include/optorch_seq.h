/*
 * optorch_seq -- one training step of a sequential CNN split into k checkpointed
 * segments, for AMD MI355X (gfx950).  C ABI; no C++ or framework types cross it.
 *
 * Method (paper, Introduction, paragraph on sequential models, and Section
 * "Sequential-checkpoint training"): a sequential network is run as a list of
 * segments; every segment except the last runs without keeping its intermediate
 * activations, only the input of each segment is kept, and during back-propagation
 * each such segment's forward pass is run again from its kept input to rebuild the
 * activations its backward pass needs.  Section "Mixed-precision training": 16-bit
 * storage with 32-bit arithmetic where stability needs it; here that means fp32
 * master weights, fp16/bf16 activations and weight copies, fp32 accumulation, and a
 * dynamic loss scale.  Section "Discussion & Recommendation": checkpoints are
 * cheapest at narrow layers -- the byte-aware plan mode below.
 *
 * Memory ownership: the handle owns host memory only.  Both device arenas are
 * allocated by the caller (sizes from optorch_seq_query) and borrowed until
 * optorch_seq_destroy; the library sub-allocates the activation arena itself, which
 * is what makes the reported peak byte counts exact.  All kernels are enqueued on
 * the stream given to optorch_seq_bind; optorch_seq_step synchronises that stream
 * once, at its end, to read back the loss and the overflow flag.
 *
 * Error behaviour: every int-returning function returns OPTORCH_OK (0) or a negative
 * code; optorch_seq_last_error gives a message for the most recent failure on that
 * handle (or, with a NULL handle, for the most recent failed create on this thread).
 * A step skipped because of a non-finite gradient is a success with *step_skipped = 1.
 * A handle is not thread-safe.
 */
#ifndef OPTORCH_SEQ_H
#define OPTORCH_SEQ_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct optorch_seq optorch_seq_t; /* opaque */

enum { OPTORCH_OK = 0,
       OPTORCH_E_INVALID = -1,  /* bad argument or unsupported layer combination            */
       OPTORCH_E_BUDGET = -2,   /* planned arena exceeds the budget or the bound arena      */
       OPTORCH_E_HIP = -3,      /* HIP runtime error                                        */
       OPTORCH_E_ORDER = -4 };  /* wrong call order (e.g. step before bind / set_params)    */

typedef enum { OPTORCH_FP32 = 0, OPTORCH_BF16 = 1, OPTORCH_FP16 = 2 } optorch_precision_t;

/* A unit is the atomic piece a segment boundary may fall between (a residual block's
 * skip connection never crosses a boundary). */
typedef enum {
  OPTORCH_CONV = 0,             /* conv ksize x ksize [+bias] [+BatchNorm] [+ReLU]                        */
  OPTORCH_MAXPOOL2 = 1,         /* 2x2 max-pool, stride 2                                                 */
  OPTORCH_BASIC_BLOCK = 2,      /* conv3x3(stride)-BN-ReLU, conv3x3-BN, + shortcut, ReLU                  */
  OPTORCH_BOTTLENECK = 3,       /* conv1x1-BN-ReLU, conv3x3(stride)-BN-ReLU, conv1x1-BN, + shortcut, ReLU */
  OPTORCH_GAP_LINEAR_CE = 4,    /* global average pool, linear (+bias), mean softmax cross-entropy        */
  OPTORCH_FLATTEN_LINEAR_CE = 5 /* NHWC flatten, linear (+bias), mean softmax cross-entropy               */
} optorch_unit_kind_t;

/* Plain data, caller-owned, copied by create.  For blocks cin/cout are the block's input
 * and output channels (bottleneck width = cout/4) and the shortcut is the identity when
 * cin == cout and stride == 1, else conv1x1(stride)+BN.  For the two head kinds cin is the
 * channel count of the incoming map and cout the number of classes.  ksize is 1 or 3,
 * stride 1 or 2. */
typedef struct {
  int32_t kind, cin, cout, ksize, stride, pad;
  int32_t has_bn, has_relu, has_bias, reserved;
} optorch_unit_t;

typedef struct {
  int32_t k_segments;              /* >= 1; 1 = every activation stored (no recomputation);
                                      0 = chosen by create: the fewest segments whose planned
                                      activation arena fits activation_budget_bytes                */
  const int32_t* boundaries;       /* NULL: the planner chooses; else k-1 ascending unit indices,
                                      segment j starts at unit boundaries[j-1]                    */
  int32_t plan_mode;               /* 0 = equal unit count (remainder joins the last segment),
                                      1 = minimise peak saved bytes over contiguous partitions,
                                      2 = least recomputation (the last segment is not replayed)
                                          among the partitions within the minimum peak of mode 1,
                                          or within activation_budget_bytes when that is set       */
  int32_t precision;               /* optorch_precision_t                                         */
  int32_t batch, height, width, channels, num_classes;
  uint64_t activation_budget_bytes; /* 0 = unlimited; create fails with OPTORCH_E_BUDGET if the
                                       planned activation arena is larger                         */
  float momentum;                  /* SGD momentum (0 = plain SGD)                                */
  float bn_eps;                    /* <= 0 selects 1e-5                                           */
  float bn_momentum;               /* running-statistics momentum; <= 0 selects 0.1               */
  float loss_scale_init;           /* <= 0 selects 1 (fp32, bf16) or 65536 (fp16)                 */
  float scale_growth;              /* <= 0 selects 2                                              */
  float scale_backoff;             /* <= 0 selects 0.5                                            */
  int32_t growth_interval;         /* <= 0 selects 2000 (fp16) or "never" (fp32, bf16)            */
  int32_t storage_mode;            /* what a conv-BatchNorm-ReLU keeps for backward: 0 = its pre-
                                      normalisation output Z and its activation A; 1 = Z only where
                                      A = ReLU(BN(Z)) has no skip connection added: backward rebuilds
                                      such an A with one elementwise pass right before its first use
                                      (fewer saved bytes, one more pass over Z per layer; gradients
                                      bit-identical to mode 0); -1 = chosen by create: 0 if the arena
                                      then fits activation_budget_bytes, else 1 (tried before a
                                      further segment, which costs more time).  In modes 0 and 1 an A
                                      inside a unit whose only reader is a convolution that can apply
                                      the BatchNorm itself while loading Z (16-bit 1x1 layers) is
                                      never written at all, in forward or backward; 2 = as mode 0 but
                                      every A is written and kept (same bits; the layout the other
                                      modes are checked against)                                   */
} optorch_seq_config_t;

/* Plans the step on the host: expands units into kernels, chooses segment boundaries,
 * assigns every activation an offset in the activation arena and builds the static launch
 * schedule (forward of segments 0..k-2 keeping only their inputs, forward of the last segment
 * keeping what its backward needs, then per segment in reverse: replay + backward).  Touches
 * no device.  units: host pointer, n_units entries, the last one a head kind. */
int optorch_seq_create(const optorch_unit_t* units, int32_t n_units,
                       const optorch_seq_config_t* cfg, optorch_seq_t** out);

/* Sizes the caller needs (any out pointer may be NULL).
 *   param_count               number of fp32 parameters in the flat parameter vector
 *   param_arena_bytes         bytes of device memory for the parameter arena (master weights,
 *                             momentum, gradients, 16-bit copies, BN running statistics, flags)
 *   act_arena_bytes           bytes of device memory for the activation arena (= planned peak)
 *   planned_peak_saved_bytes  planned peak of live checkpoints + tensors kept for backward
 *   boundaries_out            k-1 unit indices (host) */
int optorch_seq_query(const optorch_seq_t* h, uint64_t* param_count, uint64_t* param_arena_bytes,
                      uint64_t* act_arena_bytes, uint64_t* planned_peak_saved_bytes,
                      int32_t* boundaries_out);

/* Lends the two device arenas (256-byte aligned device pointers) and the HIP stream
 * (hipStream_t, NULL = default stream) to the handle. */
int optorch_seq_bind(optorch_seq_t* h, void* param_arena_dev, uint64_t param_arena_bytes,
                     void* act_arena_dev, uint64_t act_arena_bytes, void* hip_stream);

/* Copies n = param_count fp32 values (flat order: unit order; inside a unit conv weight
 * (C_out, kh, kw, C_in), [bias], BN gamma, BN beta; inside a block conv1, conv2, [conv3], then the
 * projection shortcut; linear weight (classes x features), bias) from host (is_device = 0) or
 * device memory, zeroes the momentum, resets BN running statistics and the loss scale, and
 * refreshes the 16-bit copies. */
int optorch_seq_set_params(optorch_seq_t* h, const float* src, uint64_t n, int32_t is_device);
int optorch_seq_get_params(const optorch_seq_t* h, float* dst, uint64_t n, int32_t is_device);

/* One training step on one batch.
 *   x_dev             device, batch x height x width x channels fp32, NHWC
 *   y_dev             device, batch int32 labels in [0, num_classes)
 *   lr                learning rate of this step
 *   loss_out          host, mean softmax cross-entropy of the batch (unscaled)
 *   grads_dev         device or NULL: receives param_count fp32 gradients, unscaled, w.r.t. the
 *                     weights used in this step's forward; unspecified on a skipped step
 *   peak_saved_bytes  host or NULL: observed peak of checkpoints + tensors kept for backward
 *   peak_arena_bytes  host or NULL: high-water mark of the activation arena
 *   loss_scale_out    host or NULL: loss scale after this step
 *   step_skipped      host or NULL: 1 if a non-finite gradient was found (weights untouched,
 *                     scale multiplied by scale_backoff), else 0
 * A label outside [0, num_classes) is found on the device before the forward pass: the call returns
 * OPTORCH_E_INVALID after the step's kernels have run, with the master weights, momentum, 16-bit copies, BatchNorm
 * running statistics, loss scale and the out arguments untouched; the activation arena and grads_dev are then
 * unspecified. */
int optorch_seq_step(optorch_seq_t* h, const float* x_dev, const int32_t* y_dev, float lr,
                     float* loss_out, float* grads_dev, uint64_t* peak_saved_bytes,
                     uint64_t* peak_arena_bytes, float* loss_scale_out, int32_t* step_skipped);

/* For callers that cannot allocate device memory where they step (code under HIP graph capture, tight serving or
 * training loops, harnesses that forbid allocation): optorch_seq_step with the activation arena -- checkpoints, tensors
 * kept for backward, transients, partial sums of the split reductions -- taken from a device array that the library
 * holds statically, OPTORCH_STATIC_ARENA_BYTES on every GPU it runs on until the process ends, instead of from the
 * activation arena given to optorch_seq_bind (which this call does not touch; the parameter arena, the stream and the
 * pinned read-back buffer are the bound ones).  The call allocates nothing, on the device or through any library.
 * OPTORCH_E_BUDGET if the planned activation arena (optorch_seq_query) is larger than the static one; OPTORCH_E_ORDER
 * while launch timing is enabled.  The array is shared by every handle and call on that GPU and keeps the previous
 * call's contents; no kernel of the step reads arena memory it has not written in the same step, so nothing has to be
 * cleared -- but two such calls that overlap on one GPU (different streams or threads) race.  Arguments, results and
 * all other errors as optorch_seq_step, to which the results are bit-identical. */
#define OPTORCH_STATIC_ARENA_BYTES (32u << 20)
int optorch_seq_step_static(optorch_seq_t* h, const float* x_dev, const int32_t* y_dev, float lr, float* loss_out,
                            float* grads_dev, uint64_t* peak_saved_bytes, uint64_t* peak_arena_bytes,
                            float* loss_scale_out, int32_t* step_skipped);

/* optorch_seq_step on a batch that arrives encoded (paper, Section "Image Data-flow Optimization": the network's
 * first layer decodes).  a_dev is the batch in the form optorch_encode of optorch_dataflow.h produces for groups of z
 * images of height x width x channels 8-bit pixels: device, uint64 [ceil(batch / z)][height * width * channels][words].
 * The step's first kernel is Algorithm "Decode" fused with pixel * scale[c] + shift[c] (fp32, one fused multiply-add)
 * and the cast to the storage type; it takes the place of the cast of an fp32 batch, and everything after it is
 * optorch_seq_step.  scale_host / shift_host: `channels` floats each, host memory, read during the call; the
 * network's input must have at most 16 channels; 1 <= z <= 16.  Other arguments and errors as optorch_seq_step. */
int optorch_seq_step_encoded(optorch_seq_t* h, const uint64_t* a_dev, int32_t z, const float* scale_host,
                             const float* shift_host, const int32_t* y_dev, float lr, float* loss_out,
                             float* grads_dev, uint64_t* peak_saved_bytes, uint64_t* peak_arena_bytes,
                             float* loss_scale_out, int32_t* step_skipped);

/* Inference with the network as it stands (the counterpart of training-mode BatchNorm; the paper evaluates its
 * trained networks, Section "Results"): the forward pass of every segment, nothing kept, with
 * each BatchNorm using its running mean and variance instead of the batch statistics, up to the logits.
 *   x_dev       device: batch x height x width x channels fp32, NHWC (the batch size of create)
 *   logits_dev  device: receives batch x num_classes fp32
 * Runs on the bound stream and returns after it has finished.  Uses the activation arena: not concurrently with
 * optorch_seq_step on the same handle.  Errors as optorch_seq_step. */
int optorch_seq_predict(optorch_seq_t* h, const float* x_dev, float* logits_dev);

/* optorch_seq_predict on a batch in encoded form; a_dev, z, scale_host and shift_host as for
 * optorch_seq_step_encoded. */
int optorch_seq_predict_encoded(optorch_seq_t* h, const uint64_t* a_dev, int32_t z, const float* scale_host,
                                const float* shift_host, float* logits_dev);

/* Inspection of the forward pass (for parity tests unit by unit; not part of a training loop): runs the forward
 * entries of the step's static schedule on x_dev exactly as optorch_seq_step runs them (batch statistics in every
 * BatchNorm, the segments' keep / discard rules, the same kernels and launch shapes), stops after the entry that writes
 * the output activation of body unit `unit`, and converts that tensor from the storage type to fp32 into out_dev.
 * Changes no training state: weights, momentum, running statistics and loss scale are untouched.  Allocates nothing;
 * uses the bound activation arena (not concurrently with a step) and returns after the stream has finished.
 *   out_dev     device, or NULL to query *count and shape_nhwc only
 *   capacity    floats out_dev can hold; OPTORCH_E_INVALID if fewer than *count
 *   count       host or NULL: elements of the unit's output
 *   shape_nhwc  host int32[4] or NULL: batch, height, width, channels of the unit's output
 * OPTORCH_E_INVALID also if the plan fuses the unit's output into the next unit so that it is never written (a
 * convolution whose activation is only read by the max-pool behind it). */
int optorch_seq_debug_unit_output(optorch_seq_t* h, const float* x_dev, int32_t unit, float* out_dev, uint64_t capacity,
                                  uint64_t* count, int32_t* shape_nhwc);

/* The BatchNorm running statistics: for every BatchNorm in parameter order, C running means then C running
 * variances (fp32).  They start at 0 and 1 (optorch_seq_set_params) and every optorch_seq_step moves them by
 * bn_momentum towards the batch mean and the unbiased batch variance, also on a step that is then skipped for a
 * non-finite gradient (the forward pass has run by then).
 *   dst       host or device (is_device), or NULL to query the size only
 *   capacity  floats dst can hold; OPTORCH_E_INVALID if fewer than *count
 *   count     host or NULL: receives the number of floats */
int optorch_seq_running_stats(const optorch_seq_t* h, float* dst, uint64_t capacity, uint64_t* count, int32_t is_device);

/* The plan create settled on: number of segments and storage mode (the configuration's values unless they asked
 * for the automatic choice).  optorch_seq_query's boundaries_out then has *k_segments - 1 entries. */
int optorch_seq_plan_info(const optorch_seq_t* h, int32_t* k_segments, int32_t* storage_mode);

/* Number of kernel launches in one step's static schedule, and how many of them belong to the
 * replay (recomputation) of non-last segments. */
int optorch_seq_schedule_info(const optorch_seq_t* h, int32_t* n_launch_records, int32_t* n_replay_records);

/* Per-kernel-class timing for roofline figures.  While enabled, every kernel launch of optorch_seq_step carries a
 * start and a stop HIP event of its own (time stamps of the dispatch itself, i.e. the kernel's duration as a kernel
 * trace reports it); nothing is read back until optorch_seq_profile_read.
 * Classes are indexed by optorch_kernel_class_t.  For each class the read returns, summed over all profiled
 * steps since the last enable: kernel launches, schedule entries, GPU milliseconds (sum of the launches' durations),
 * algorithmic FLOPs (convolutions: 2 x output pixels x C_out x kh x kw x C_in for each of forward, data gradient
 * and weight gradient; 0 for the memory-bound classes) and algorithmic HBM bytes (every operand read once, every
 * result written once, at the storage type).  All out pointers are host arrays of OPTORCH_N_KERNEL_CLASSES. */
typedef enum {
  OPTORCH_K_CAST_IN = 0, OPTORCH_K_CONV_FWD = 1, OPTORCH_K_CONV_DGRAD = 2, OPTORCH_K_CONV_WGRAD = 3,
  OPTORCH_K_BN_STATS = 4, OPTORCH_K_BN_APPLY = 5, OPTORCH_K_BN_BWD = 6, OPTORCH_K_POOL = 7, OPTORCH_K_HEAD = 8,
  OPTORCH_K_RELU_BIAS_BWD = 9, OPTORCH_K_OPTIMIZER = 10,
  /* 1x1 convolutions apart from the others: their arithmetic intensity (C_in * C_out / (C_in + C_out) FLOP per byte at
   * best) puts them under the HBM roof, where the 3x3 layers of 128 channels and more sit under the matrix-core roof */
  OPTORCH_K_CONV1X1_FWD = 11, OPTORCH_K_CONV1X1_DGRAD = 12, OPTORCH_K_CONV1X1_WGRAD = 13, OPTORCH_N_KERNEL_CLASSES = 14
} optorch_kernel_class_t;
int optorch_seq_profile_enable(optorch_seq_t* h, int32_t enable);
/* Restricts the timing to the classes whose bit (1u << optorch_kernel_class_t) is set in class_mask; all
 * classes by default.  A timed launch costs host and GPU front-end time (about 5 us), so timing one class
 * perturbs a step far less than timing all of them.  Takes effect from the next step; call optorch_seq_profile_enable to reset the sums. */
int optorch_seq_profile_select(optorch_seq_t* h, uint32_t class_mask);
int optorch_seq_profile_read(optorch_seq_t* h, int32_t* steps, uint64_t* launches, uint64_t* entries, double* gpu_ms,
                             double* flops, double* bytes);

/* The same timing per schedule entry (one entry = one operation of one unit in one phase; live entries only, in
 * launch order).  capacity: length of the host out arrays; *n receives the number of entries (it may exceed
 * capacity, then only the first `capacity` are written).  kind: optorch_kernel_class_t; phase: 0 forward without
 * keeping, 1 forward of the last segment, 2 replay, 3 backward; gpu_ms, flops, bytes: sums over the profiled steps. */
int optorch_seq_profile_read_entries(optorch_seq_t* h, int32_t capacity, int32_t* n, int32_t* kind, int32_t* unit,
                                     int32_t* phase, double* gpu_ms, double* flops, double* bytes);

const char* optorch_seq_last_error(const optorch_seq_t* h);
void optorch_seq_destroy(optorch_seq_t* h);

#ifdef __cplusplus
}
#endif
#endif /* OPTORCH_SEQ_H */
