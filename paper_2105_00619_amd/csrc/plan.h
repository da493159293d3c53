// Host-side planning of the checkpointed training step: expansion of units into
// kernel-level operations, choice of segment boundaries, the static schedule
// (forward without keeping intermediates, forward of the last segment, then per
// segment in reverse: replay + backward), tensor lifetimes and offsets in the
// activation arena.  Pure host code; nothing here touches a device.
//
// Paper: Introduction (segments; inputs of segments are kept; all segments but the
// last discard intermediates) and Section "Sequential-checkpoint training" (the
// forward pass is run again from the previous checkpoint during back-propagation).
#pragma once
#include <cstdint>
#include <string>
#include <vector>

#include "optorch_seq.h"

namespace oseq {

constexpr uint64_t kAlign = 256;
inline uint64_t align_up(uint64_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

// A tensor of the forward graph (one per value of the network, independent of how many
// times the schedule materialises it).
struct LTensor {
  int64_t n = 0, h = 0, w = 0, c = 0;
  int esize = 4;          // bytes per element
  uint64_t bytes = 0;     // exact, unpadded
  bool needs_grad = true; // false for the network input
  int unit = -1;          // unit that produces it (-1: network input)
};

enum FKind { F_CAST_IN, F_CONV, F_BN_STATS, F_BN_APPLY, F_POOL, F_HEAD };

enum ConvAlgo { ALGO_DIRECT = 0, ALGO_MFMA = 1, ALGO_SMALLC = 2 };

// One forward operation of the network.
struct FOp {
  FKind kind = F_CONV;
  int unit = -1;
  int x = -1, skip = -1, stats = -1, out = -1;  // LTensor ids
  int mask = -1;  // F_BN_APPLY with a skip connection: LTensor of the ReLU decisions, one bit per element (one byte per
                  // 16 bytes of the output), which the backward pass reads instead of the output itself; -1: none
  int fold = 0;       // F_BN_APPLY: 1 = never run; the one convolution that reads its output applies scale, shift and
                      // ReLU to z while it stages its operand (forward and weight gradient), so the output is never stored
  int fold_src = -1;  // F_CONV: the folded F_BN_APPLY operation its input comes from, or -1
  int aux[3] = {-1, -1, -1};                     // head: feat, logits, dlogits
  int N = 0, H = 0, W = 0, C = 0, K = 0, R = 1, S = 1, stride = 1, pad = 0, P = 0, Q = 0;
  int relu = 0, has_bias = 0, has_bn = 0;
  int64_t w_off = -1, b_off = -1, gamma_off = -1, beta_off = -1;  // element offsets, flat parameter vector
  int64_t rs_off = -1;       // element offset of (running mean, running var) in the running-stat block
  int gap = 0, feat_dim = 0, classes = 0;
  int fwd_algo = ALGO_DIRECT, dgrad_algo = ALGO_DIRECT, wgrad_algo = ALGO_DIRECT;
  int wgrad_splits = 1;      // fixed by shape only: deterministic split of the pixel reduction
  int fwd_splits = 1, dgrad_splits = 1;  // fixed by shape only: deterministic split of the GEMM depth
  int red_blocks = 1;        // row blocks of the per-channel reductions (BN statistics, BN backward)
  int stat_blocks = 0;       // > 0: the convolution's forward kernel also writes per-block channel sums for the
                             // BatchNorm that follows (that many row blocks); set on the conv and on its F_BN_STATS
  int stat_fold = 0;         // rows into which the finishing step first folds those block sums (0: none); extra workspace
};

enum SKind {
  S_CAST_IN, S_CONV_FWD, S_BN_STATS, S_BN_APPLY, S_POOL_FWD, S_HEAD_FWD,
  S_HEAD_BWD, S_BN_BWD, S_RELU_BWD, S_BIAS_GRAD, S_WGRAD, S_DGRAD, S_POOL_BWD
};
enum Phase { PH_FWD_NOSAVE = 0, PH_FWD_LAST = 1, PH_REPLAY = 2, PH_BWD = 3 };

// One materialisation of a tensor in the activation arena.
struct Inst {
  int logical = -1;       // LTensor id, or -1 for workspaces
  uint64_t bytes = 0;
  int def_op = -1, last_use = -1;
  uint64_t offset = 0;
  bool fwd_value = false; // produced by a forward-kind operation
  bool held = false;      // checkpoint or kept for backward (counts as "saved")
  bool allocated = false;
};

// One entry of the static schedule.
struct SOp {
  SKind kind = S_CONV_FWD;
  int fop = -1;
  int phase = 0, seg = 0;
  int in[4] = {-1, -1, -1, -1};
  int out[4] = {-1, -1, -1, -1};
  int variant = 0;  // S_BN_BWD: 1 = in[0] is the gradient of the 2x2 max-pool behind the activation (pooled size);
                    // 2 = in[3] is a bit mask of ReLU decisions (FOp::mask) to apply to in[0], not an activation.
                    // S_DGRAD: in[2] >= 0 is such a mask for the addend in[1]
                    // S_CONV_FWD with in[1] >= 0, S_WGRAD with in[2] >= 0: in[0] is the z of a folded BatchNorm apply
                    // and that slot its statistics tensor (FOp::fold_src)
  bool live = true;
};

struct Plan {
  // inputs
  std::vector<optorch_unit_t> units;
  optorch_seq_config_t cfg{};
  int esize = 4;  // bytes per activation element
  // forward graph
  std::vector<LTensor> tensors;
  std::vector<FOp> fops;
  std::vector<int> unit_first_fop, unit_last_fop;  // [unit] range of fops (inclusive first, exclusive last)
  std::vector<int> unit_in, unit_out;              // [unit] LTensor ids
  uint64_t n_params = 0;
  uint64_t n_running = 0;  // floats of BN running statistics
  // partition
  std::vector<int> seg_begin;  // k+1 entries, unit indices
  // schedule
  std::vector<Inst> insts;
  std::vector<SOp> sched;
  uint64_t arena_bytes = 0;       // high-water mark of the activation arena (aligned offsets)
  uint64_t peak_saved_bytes = 0;  // exact tensor sizes, no alignment
  uint64_t peak_live_bytes = 0;   // all live tensors incl. transients, exact sizes
  int n_launches = 0, n_replay_launches = 0;
  std::string error;
};

// Builds the forward graph from the unit list.  Returns false and sets plan.error on failure.
bool build_graph(Plan& p);
// Chooses segment boundaries (explicit, equal count, or min peak) into plan.seg_begin.
bool choose_segments(Plan& p);
// Builds schedule, lifetimes, offsets and peak figures for plan.seg_begin.
bool build_schedule(Plan& p);
// Peak saved bytes of the partition given by seg_begin, from the closed form
//   max_j ( sum_{i<=j} checkpoint_i + saved_j ),
// with per-unit saved bytes taken from the all-stored schedule.  Used by the min-peak planner.
uint64_t model_peak_saved(const Plan& p, const std::vector<int>& seg_begin);

int launches_of(const SOp& op, const FOp& f);

}  // namespace oseq
