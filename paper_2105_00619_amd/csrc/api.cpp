// C ABI of the checkpointed training step: plan on create, borrow device arenas on bind, walk the static
// schedule on step.  See include/optorch_seq.h for the contract of every entry point.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstring>
#include <new>
#include <string>
#include <vector>

#include "kernels.h"
#include "launch.h"
#include "optorch_seq.h"
#include "plan.h"

using namespace oseq;

namespace oseq {
thread_local LaunchTimer g_launch_timer;
}

struct optorch_seq {
  Plan plan;
  char* pbase = nullptr; uint64_t pbytes = 0;
  char* abase = nullptr; uint64_t abytes = 0;
  hipStream_t stream = nullptr;
  uint64_t off_w = 0, off_v = 0, off_g = 0, off_h = 0, off_wt = 0, off_run = 0, off_scal = 0, param_arena_bytes = 0;
  bool bound = false, params_set = false;
  bool x_encoded = false;  // the current step's batch came in encoded form
  int dt = 0, in_channels = 0;
  float scale = 1.f, scale_init = 1.f, growth = 2.f, backoff = 0.5f, eps = 1e-5f, bn_mom = 0.1f, momentum = 0.f;
  int growth_interval = 0, clean = 0;
  bool dynamic_scale = false;
  float* host_rb = nullptr;  // pinned read-back buffer: loss + flags
  std::vector<TransposeJob> transpose_jobs;  // layers whose data gradient reads a transposed weight copy
  mutable std::string err;
  // profiling: an event pair per kernel launch of the timed entries, harvested on read
  bool profiling = false;
  uint32_t prof_mask = 0xffffffffu;  // kernel classes whose launches are timed
  std::vector<hipEvent_t> ev_pool;
  size_t ev_used = 0;
  std::vector<int> ev_class;  // class of pair i
  std::vector<int> ev_entry;  // schedule index of pair i (-1: optimizer)
  std::vector<double> entry_ms;  // per schedule entry
  int prof_steps = 0;
  uint64_t prof_launches[OPTORCH_N_KERNEL_CLASSES] = {0}, prof_entries[OPTORCH_N_KERNEL_CLASSES] = {0};
  double prof_ms[OPTORCH_N_KERNEL_CLASSES] = {0}, prof_flops[OPTORCH_N_KERNEL_CLASSES] = {0},
         prof_bytes[OPTORCH_N_KERNEL_CLASSES] = {0};
};

static thread_local std::string g_create_error;

static int set_err(const optorch_seq_t* h, int code, const std::string& m) { h->err = m; return code; }

static int hip_fail(const optorch_seq_t* h, hipError_t e, const char* what) {
  return set_err(h, OPTORCH_E_HIP, std::string(what) + ": " + hipGetErrorString(e));
}

// refresh the transposed weight copies the data-gradient GEMMs read (after every change of the master weights)
static void refresh_transposed_weights(optorch_seq_t* h) {
  if (!h->transpose_jobs.empty())
    launch_weight_transposes(h->stream, h->dt, (const float*)(h->pbase + h->off_w), h->pbase + h->off_wt,
                             h->transpose_jobs.data(), (int)h->transpose_jobs.size());
}

extern "C" int optorch_seq_create(const optorch_unit_t* units, int32_t n_units, const optorch_seq_config_t* cfg,
                                  optorch_seq_t** out) {
  if (out) *out = nullptr;
  if (!units || !cfg || !out || n_units < 1) { g_create_error = "null argument or empty unit list"; return OPTORCH_E_INVALID; }
  optorch_seq_t* h = new (std::nothrow) optorch_seq();
  if (!h) { g_create_error = "out of host memory"; return OPTORCH_E_INVALID; }
  Plan& p = h->plan;
  p.units.assign(units, units + n_units);
  p.cfg = *cfg;
  if (p.cfg.storage_mode == -1) p.cfg.storage_mode = 0;  // chosen below
  std::vector<int32_t> bcopy;
  if (cfg->boundaries && cfg->k_segments > 1) {
    bcopy.assign(cfg->boundaries, cfg->boundaries + (cfg->k_segments - 1));
    p.cfg.boundaries = bcopy.data();
  } else {
    p.cfg.boundaries = nullptr;
  }
  bool ok = build_graph(p);
  if (ok) {  // kernel choice per convolution, from the layer shape only (never from k or from free memory)
    for (FOp& f : p.fops)
      if (f.kind == F_CONV) {
        const ConvGeom g{f.N, f.H, f.W, f.C, f.K, f.R, f.S, f.stride, f.pad, f.P, f.Q};
        const int dt = cfg->precision;
        f.fwd_algo = conv_mfma_fwd_ok(dt, g) ? ALGO_MFMA : conv_smallc_fwd_ok(g) ? ALGO_SMALLC : ALGO_DIRECT;
        f.dgrad_algo = conv_mfma_dgrad_ok(dt, g) ? ALGO_MFMA : ALGO_DIRECT;
        f.wgrad_algo = conv_mfma_wgrad_ok(dt, g) ? ALGO_MFMA : conv_smallc_wgrad_ok(g) ? ALGO_SMALLC : ALGO_DIRECT;
        if (f.fwd_algo == ALGO_MFMA) f.fwd_splits = conv_mfma_fwd_splits(dt, g);
        if (f.dgrad_algo == ALGO_MFMA) f.dgrad_splits = conv_mfma_dgrad_splits(dt, g);
        if (f.wgrad_algo == ALGO_MFMA) f.wgrad_splits = conv_mfma_wgrad_splits(dt, g);
        if (f.wgrad_algo == ALGO_SMALLC) f.wgrad_splits = conv_smallc_wgrad_splits(g);
        if (f.has_bn && f.fwd_algo == ALGO_MFMA) f.stat_blocks = conv_mfma_fwd_stat_blocks(dt, g);
      }
    // the BatchNorm statistics operation that follows such a convolution only runs its finishing kernel
    for (size_t i = 0; i + 1 < p.fops.size(); ++i)
      if (p.fops[i].kind == F_CONV && p.fops[i].stat_blocks > 0 && p.fops[i + 1].kind == F_BN_STATS &&
          p.fops[i + 1].x == p.fops[i].out)
        p.fops[i + 1].stat_blocks = p.fops[i].stat_blocks, p.fops[i].stat_fold = p.fops[i + 1].stat_fold = bn_stats_fold_rows(p.fops[i].stat_blocks);
      else if (p.fops[i].kind == F_CONV)
        p.fops[i].stat_blocks = 0;
    // A BatchNorm apply + ReLU without a skip connection whose output has one reader, a convolution of the same unit
    // whose forward and weight-gradient kernels can do it themselves, is folded into that convolution: the activation
    // is never written (storage mode 2 keeps every activation instead).  From the network and the layer shapes only.
    // (A BatchNorm without ReLU keeps its apply launch: the folding kernels always apply the ReLU.)
    if (p.cfg.storage_mode != 2) {
      std::vector<int> readers(p.tensors.size(), 0), reader(p.tensors.size(), -1);
      for (size_t i = 0; i < p.fops.size(); ++i) {
        const FOp& f = p.fops[i];
        if (f.x >= 0) { ++readers[f.x]; reader[f.x] = (int)i; }
        if (f.skip >= 0) { ++readers[f.skip]; reader[f.skip] = (int)i; }
      }
      for (size_t i = 0; i < p.fops.size(); ++i) {
        FOp& b = p.fops[i];
        if (b.kind != F_BN_APPLY || !b.relu || b.skip >= 0 || b.mask >= 0 || readers[b.out] != 1) continue;
        FOp& cv = p.fops[reader[b.out]];
        if (cv.kind != F_CONV || cv.x != b.out || cv.unit != b.unit) continue;
        if (cv.fwd_algo != ALGO_MFMA || cv.wgrad_algo != ALGO_MFMA) continue;
        const ConvGeom g{cv.N, cv.H, cv.W, cv.C, cv.K, cv.R, cv.S, cv.stride, cv.pad, cv.P, cv.Q};
        if (!conv_fold_fwd_ok(cfg->precision, g) || !conv_fold_wgrad_ok(cfg->precision, g)) continue;
        b.fold = 1;
        cv.fold_src = (int)i;
      }
    }
    // k_segments 0 and storage_mode -1 leave the choice to the plan: the cheapest candidate in step time whose
    // arena fits the budget -- fewest segments first (each further segment replays more of the forward pass),
    // and at equal segments keeping activations before rebuilding them
    const bool auto_k = cfg->k_segments == 0, auto_mode = cfg->storage_mode == -1;
    if (auto_k && cfg->boundaries) { p.error = "explicit boundaries need k_segments"; ok = false; }
    const int k_lo = auto_k ? 1 : cfg->k_segments, k_hi = auto_k ? n_units : cfg->k_segments;
    bool fits = false;
    uint64_t least = ~0ull;  // smallest arena among the candidates tried
    for (int k = k_lo; ok && !fits && k <= k_hi; ++k)
      for (int mode = auto_mode ? 0 : cfg->storage_mode; ok && !fits && mode <= (auto_mode ? 1 : cfg->storage_mode); ++mode) {
        p.cfg.k_segments = k;
        p.cfg.storage_mode = mode;
        ok = choose_segments(p) && build_schedule(p);
        fits = ok && (!cfg->activation_budget_bytes || p.arena_bytes <= cfg->activation_budget_bytes);
        if (ok && p.arena_bytes < least) least = p.arena_bytes;
      }
    if (ok && !fits && (auto_k || auto_mode)) {
      g_create_error = "no plan fits the budget of " + std::to_string(cfg->activation_budget_bytes) +
                       " bytes: the smallest activation arena among the candidates is " + std::to_string(least) + " bytes";
      delete h;
      return OPTORCH_E_BUDGET;
    }
  }
  p.cfg.boundaries = nullptr;  // the copy dies with this call; seg_begin holds the result
  if (!ok) { g_create_error = p.error; delete h; return OPTORCH_E_INVALID; }
  if (cfg->activation_budget_bytes && p.arena_bytes > cfg->activation_budget_bytes) {
    g_create_error = "planned activation arena of " + std::to_string(p.arena_bytes) + " bytes exceeds the budget of " +
                     std::to_string(cfg->activation_budget_bytes) + " bytes";
    delete h;
    return OPTORCH_E_BUDGET;
  }
  h->dt = cfg->precision;
  h->in_channels = cfg->channels;
  h->eps = cfg->bn_eps > 0 ? cfg->bn_eps : 1e-5f;
  h->bn_mom = cfg->bn_momentum > 0 ? cfg->bn_momentum : 0.1f;
  h->momentum = cfg->momentum;
  h->growth = cfg->scale_growth > 0 ? cfg->scale_growth : 2.f;
  h->backoff = cfg->scale_backoff > 0 ? cfg->scale_backoff : 0.5f;
  h->scale_init = cfg->loss_scale_init > 0 ? cfg->loss_scale_init : (cfg->precision == OPTORCH_FP16 ? 65536.f : 1.f);
  h->growth_interval = cfg->growth_interval > 0 ? cfg->growth_interval : (cfg->precision == OPTORCH_FP16 ? 2000 : 0);
  h->dynamic_scale = h->growth_interval > 0;
  h->scale = h->scale_init;
  const uint64_t P = p.n_params;
  uint64_t o = 0;
  h->off_w = o; o = align_up(o + P * 4);
  h->off_v = o; o = align_up(o + P * 4);
  h->off_g = o; o = align_up(o + P * 4);
  h->off_h = o; if (h->dt != DT_F32) o = align_up(o + P * 2);
  h->off_wt = o; o = align_up(o + P * p.esize);  // transposed conv weights for the data-gradient GEMM
  h->off_run = o; o = align_up(o + p.n_running * 4);
  h->off_scal = o; o = align_up(o + 256);
  h->param_arena_bytes = o;
  for (const FOp& f : p.fops)
    if (f.kind == F_CONV && f.dgrad_algo == ALGO_MFMA && p.tensors[f.x].needs_grad)
      h->transpose_jobs.push_back(TransposeJob{f.w_off, f.K, f.R * f.S, f.C, 0});
  *out = h;
  return OPTORCH_OK;
}

extern "C" int optorch_seq_query(const optorch_seq_t* h, uint64_t* param_count, uint64_t* param_arena_bytes,
                                 uint64_t* act_arena_bytes, uint64_t* planned_peak_saved_bytes, int32_t* boundaries_out) {
  if (!h) return OPTORCH_E_INVALID;
  if (param_count) *param_count = h->plan.n_params;
  if (param_arena_bytes) *param_arena_bytes = h->param_arena_bytes;
  if (act_arena_bytes) *act_arena_bytes = h->plan.arena_bytes;
  if (planned_peak_saved_bytes) *planned_peak_saved_bytes = h->plan.peak_saved_bytes;
  if (boundaries_out)
    for (size_t j = 1; j + 1 < h->plan.seg_begin.size(); ++j) boundaries_out[j - 1] = h->plan.seg_begin[j];
  return OPTORCH_OK;
}

extern "C" int optorch_seq_plan_info(const optorch_seq_t* h, int32_t* k_segments, int32_t* storage_mode) {
  if (!h) return OPTORCH_E_INVALID;
  if (k_segments) *k_segments = (int32_t)h->plan.seg_begin.size() - 1;
  if (storage_mode) *storage_mode = h->plan.cfg.storage_mode;
  return OPTORCH_OK;
}

extern "C" int optorch_seq_schedule_info(const optorch_seq_t* h, int32_t* n_launch_records, int32_t* n_replay_records) {
  if (!h) return OPTORCH_E_INVALID;
  if (n_launch_records) *n_launch_records = h->plan.n_launches;
  if (n_replay_records) *n_replay_records = h->plan.n_replay_launches;
  return OPTORCH_OK;
}

extern "C" int optorch_seq_bind(optorch_seq_t* h, void* param_arena_dev, uint64_t param_arena_bytes, void* act_arena_dev,
                                uint64_t act_arena_bytes, void* hip_stream) {
  if (!h) return OPTORCH_E_INVALID;
  if (!param_arena_dev || !act_arena_dev) return set_err(h, OPTORCH_E_INVALID, "null arena pointer");
  if (((uintptr_t)param_arena_dev | (uintptr_t)act_arena_dev) & (kAlign - 1))
    return set_err(h, OPTORCH_E_INVALID, "arena pointers must be 256-byte aligned");
  if (param_arena_bytes < h->param_arena_bytes) return set_err(h, OPTORCH_E_BUDGET, "parameter arena too small");
  if (act_arena_bytes < h->plan.arena_bytes) return set_err(h, OPTORCH_E_BUDGET, "activation arena smaller than the planned peak");
  if (!h->host_rb) {
    hipError_t e = hipHostMalloc((void**)&h->host_rb, 256, hipHostMallocDefault);
    if (e != hipSuccess) return hip_fail(h, e, "hipHostMalloc");
  }
  h->pbase = (char*)param_arena_dev; h->pbytes = param_arena_bytes;
  h->abase = (char*)act_arena_dev; h->abytes = act_arena_bytes;
  h->stream = (hipStream_t)hip_stream;
  h->bound = true;
  h->params_set = false;
  return OPTORCH_OK;
}

extern "C" int optorch_seq_set_params(optorch_seq_t* h, const float* src, uint64_t n, int32_t is_device) {
  if (!h) return OPTORCH_E_INVALID;
  if (!h->bound) return set_err(h, OPTORCH_E_ORDER, "set_params before bind");
  if (!src || n != h->plan.n_params) return set_err(h, OPTORCH_E_INVALID, "set_params: wrong parameter count");
  hipStream_t st = h->stream;
  hipError_t e = hipMemcpyAsync(h->pbase + h->off_w, src, n * 4, is_device ? hipMemcpyDeviceToDevice : hipMemcpyHostToDevice, st);
  if (e != hipSuccess) return hip_fail(h, e, "hipMemcpyAsync(params)");
  launch_fill(st, (float*)(h->pbase + h->off_v), (int64_t)n, 0.f);
  launch_fill(st, (float*)(h->pbase + h->off_g), (int64_t)n, 0.f);
  // running statistics: mean 0, variance 1, per BatchNorm as (mean[C], var[C])
  for (const FOp& f : h->plan.fops)
    if (f.kind == F_BN_STATS) {
      float* r = (float*)(h->pbase + h->off_run) + f.rs_off;
      launch_fill(st, r, f.C, 0.f);
      launch_fill(st, r + f.C, f.C, 1.f);
    }
  launch_fill(st, (float*)(h->pbase + h->off_scal), 64, 0.f);
  launch_cast_params(st, h->dt, (const float*)(h->pbase + h->off_w), h->pbase + h->off_h, (int64_t)n);
  refresh_transposed_weights(h);
  e = hipStreamSynchronize(st);
  if (e != hipSuccess) return hip_fail(h, e, "hipStreamSynchronize");
  e = hipGetLastError();
  if (e != hipSuccess) return hip_fail(h, e, "set_params kernels");
  h->scale = h->scale_init; h->clean = 0;
  h->params_set = true;
  return OPTORCH_OK;
}

extern "C" int optorch_seq_get_params(const optorch_seq_t* h, float* dst, uint64_t n, int32_t is_device) {
  if (!h) return OPTORCH_E_INVALID;
  if (!h->bound || !h->params_set) return set_err(h, OPTORCH_E_ORDER, "get_params before bind/set_params");
  if (!dst || n != h->plan.n_params) return set_err(h, OPTORCH_E_INVALID, "get_params: wrong parameter count");
  hipError_t e = hipStreamSynchronize(h->stream);
  if (e != hipSuccess) return hip_fail(h, e, "hipStreamSynchronize");
  e = hipMemcpy(dst, h->pbase + h->off_w, n * 4, is_device ? hipMemcpyDeviceToDevice : hipMemcpyDeviceToHost);
  if (e != hipSuccess) return hip_fail(h, e, "hipMemcpy(params)");
  return OPTORCH_OK;
}

namespace {

struct Ctx {
  optorch_seq_t* h;
  const float* x; const int32_t* y;
  char* abase = nullptr;  // the activation arena this call works in (the bound one unless stated otherwise)
  bool touch_running = true;  // BatchNorm statistics also move the running estimates (a training step's forward)
  // the batch in encoded form instead of x (groups of xz images, Algorithm "Encode"), with the input normalisation
  const uint64_t* xa = nullptr; int xz = 0; const float* xscale = nullptr; const float* xshift = nullptr;
  void* at(int inst) const { return inst < 0 ? nullptr : (void*)(abase + h->plan.insts[inst].offset); }
  float* w32(int64_t off) const { return (float*)(h->pbase + h->off_w) + off; }
  float* g32(int64_t off) const { return (float*)(h->pbase + h->off_g) + off; }
  const void* wc(int64_t off) const {  // weights in the compute type
    return h->dt == DT_F32 ? (const void*)w32(off) : (const void*)(h->pbase + h->off_h + off * 2);
  }
  int* flags() const { return (int*)(h->pbase + h->off_scal + 64); }
  float* loss() const { return (float*)(h->pbase + h->off_scal); }
};

ConvGeom geom(const FOp& f) { return ConvGeom{f.N, f.H, f.W, f.C, f.K, f.R, f.S, f.stride, f.pad, f.P, f.Q}; }

void run_op(const Ctx& c, const SOp& s) {
  optorch_seq_t* h = c.h;
  const FOp& f = h->plan.fops[s.fop];
  hipStream_t st = h->stream;
  const int dt = h->dt;
  switch (s.kind) {
    case S_CAST_IN:
      if (c.xa)  // the decode layer as the first kernel of the step
        launch_decode_cast(st, dt, c.xa, f.N, (int64_t)f.H * f.W * f.C, c.xz, f.C, c.xscale, c.xshift, c.at(s.out[0]));
      else
        launch_cast_in(st, dt, c.x, c.at(s.out[0]), (int64_t)f.N * f.H * f.W * f.C);
      break;
    case S_CONV_FWD:
      if (f.fwd_algo == ALGO_MFMA)
        launch_conv_fwd_mfma(st, dt, c.at(s.in[0]), c.wc(f.w_off), f.has_bias ? c.w32(f.b_off) : nullptr, c.at(s.out[0]),
                             (float*)c.at(s.out[1]), (float*)c.at(s.out[2]), f.fwd_splits, geom(f), f.relu,
                             (const float*)c.at(s.in[1]));
      else if (f.fwd_algo == ALGO_SMALLC)
        launch_conv_fwd_smallc(st, dt, c.at(s.in[0]), c.wc(f.w_off), f.has_bias ? c.w32(f.b_off) : nullptr, c.at(s.out[0]),
                               geom(f), f.relu);
      else
        launch_conv_fwd_direct(st, dt, c.at(s.in[0]), c.wc(f.w_off), f.has_bias ? c.w32(f.b_off) : nullptr, c.at(s.out[0]),
                               geom(f), f.relu);
      break;
    case S_BN_STATS:
      if (s.in[1] >= 0)
        launch_bn_stats_finalize(st, (float*)c.at(s.in[1]), (int64_t)f.N * f.P * f.Q, f.C, f.stat_blocks, h->eps,
                                 h->bn_mom, c.w32(f.gamma_off), c.w32(f.beta_off), (float*)c.at(s.out[0]),
                                 c.touch_running ? (float*)(h->pbase + h->off_run) + f.rs_off : nullptr, c.flags());
      else
        launch_bn_stats(st, dt, c.at(s.in[0]), (int64_t)f.N * f.P * f.Q, f.C, f.red_blocks, (float*)c.at(s.out[1]), h->eps,
                        h->bn_mom, c.w32(f.gamma_off), c.w32(f.beta_off), (float*)c.at(s.out[0]),
                        c.touch_running ? (float*)(h->pbase + h->off_run) + f.rs_off : nullptr, c.flags());
      break;
    case S_BN_APPLY:
      if (s.out[1] >= 0)  // with the 2x2 max-pool that follows
        launch_bn_apply_pool(st, dt, c.at(s.in[0]), (const float*)c.at(s.in[1]), c.at(s.out[0]), c.at(s.out[1]), f.N, f.P,
                             f.Q, f.C, f.relu);
      else
        launch_bn_apply(st, dt, c.at(s.in[0]), (const float*)c.at(s.in[1]), c.at(s.in[2]), c.at(s.out[0]), c.at(s.out[2]),
                        (int64_t)f.N * f.P * f.Q, f.C, f.relu);
      break;
    case S_POOL_FWD:
      launch_maxpool_fwd(st, dt, c.at(s.in[0]), c.at(s.out[0]), f.N, f.H, f.W, f.C);
      break;
    case S_HEAD_FWD:
      launch_head_fwd(st, dt, c.at(s.in[0]), f.N, f.H * f.W, f.C, f.gap, f.feat_dim, f.classes, c.w32(f.w_off),
                      c.w32(f.b_off), c.y, h->scale / (float)f.N, (float*)c.at(s.out[0]), (float*)c.at(s.out[1]),
                      (float*)c.at(s.out[2]), (float*)c.at(s.out[3]), c.loss(), c.flags());
      break;
    case S_HEAD_BWD:
      launch_head_bwd(st, dt, (const float*)c.at(s.in[0]), (const float*)c.at(s.in[1]), c.w32(f.w_off), f.N, f.H * f.W, f.C,
                      f.gap, f.feat_dim, f.classes, c.g32(f.w_off), c.g32(f.b_off), (float*)c.at(s.out[1]), c.at(s.out[0]));
      break;
    case S_BN_BWD:
      if (s.variant == 1) {  // in[0] is the gradient of the max-pool behind the activation
        launch_bn_bwd_pool(st, dt, c.at(s.in[0]), c.at(s.in[1]), (const float*)c.at(s.in[2]), f.N, f.P, f.Q, f.C, f.relu,
                           f.red_blocks, (float*)c.at(s.out[2]), c.g32(f.gamma_off), c.g32(f.beta_off), c.at(s.out[0]));
        break;
      }
      // in[3]: the block output whose sign gives the ReLU decisions, or (variant 2) those decisions as a bit mask
      launch_bn_bwd(st, dt, c.at(s.in[0]), c.at(s.in[1]), s.variant == 2 ? nullptr : c.at(s.in[3]),
                    s.variant == 2 ? c.at(s.in[3]) : nullptr, (const float*)c.at(s.in[2]), (int64_t)f.N * f.P * f.Q, f.C,
                    f.relu, f.red_blocks, (float*)c.at(s.out[2]), c.g32(f.gamma_off), c.g32(f.beta_off), c.at(s.out[0]),
                    c.at(s.out[1]));
      break;
    case S_RELU_BWD:
      launch_relu_bwd(st, dt, c.at(s.in[0]), c.at(s.in[1]), c.at(s.out[0]), (int64_t)f.N * f.P * f.Q, f.K);
      break;
    case S_BIAS_GRAD:
      launch_bias_grad(st, dt, c.at(s.in[0]), (int64_t)f.N * f.P * f.Q, f.K, f.red_blocks, (float*)c.at(s.out[0]),
                       c.g32(f.b_off));
      break;
    case S_WGRAD:
      if (f.wgrad_algo == ALGO_MFMA)
        launch_conv_wgrad_mfma(st, dt, c.at(s.in[0]), c.at(s.in[1]), c.g32(f.w_off), (float*)c.at(s.out[0]), f.wgrad_splits,
                               geom(f), (const float*)c.at(s.in[2]));
      else if (f.wgrad_algo == ALGO_SMALLC)
        launch_conv_wgrad_smallc(st, dt, c.at(s.in[0]), c.at(s.in[1]), c.g32(f.w_off), (float*)c.at(s.out[0]),
                                 f.wgrad_splits, geom(f));
      else
        launch_conv_wgrad_direct(st, dt, c.at(s.in[0]), c.at(s.in[1]), c.g32(f.w_off), (float*)c.at(s.out[0]),
                                 f.wgrad_splits, geom(f));
      break;
    case S_DGRAD:
      if (f.dgrad_algo == ALGO_MFMA)
        launch_conv_dgrad_mfma(st, dt, c.at(s.in[0]), h->pbase + h->off_wt + (uint64_t)f.w_off * h->plan.esize, c.at(s.in[1]),
                               c.at(s.in[2]), c.at(s.out[0]), (float*)c.at(s.out[1]), f.dgrad_splits, geom(f));
      else
        launch_conv_dgrad_direct(st, dt, c.at(s.in[0]), c.wc(f.w_off), c.at(s.in[1]), c.at(s.out[0]), geom(f));
      break;
    case S_POOL_BWD:
      launch_maxpool_bwd(st, dt, c.at(s.in[0]), c.at(s.in[1]), c.at(s.out[0]), f.N, f.H, f.W, f.C);
      break;
  }
}

int class_of(SKind k, const FOp& f) {
  const bool pointwise = f.R == 1 && f.S == 1;
  switch (k) {
    case S_CAST_IN: return OPTORCH_K_CAST_IN;
    case S_CONV_FWD: return pointwise ? OPTORCH_K_CONV1X1_FWD : OPTORCH_K_CONV_FWD;
    case S_DGRAD: return pointwise ? OPTORCH_K_CONV1X1_DGRAD : OPTORCH_K_CONV_DGRAD;
    case S_WGRAD: return pointwise ? OPTORCH_K_CONV1X1_WGRAD : OPTORCH_K_CONV_WGRAD;
    case S_BN_STATS: return OPTORCH_K_BN_STATS;
    case S_BN_APPLY: return OPTORCH_K_BN_APPLY;
    case S_BN_BWD: return OPTORCH_K_BN_BWD;
    case S_POOL_FWD: case S_POOL_BWD: return OPTORCH_K_POOL;
    case S_HEAD_FWD: case S_HEAD_BWD: return OPTORCH_K_HEAD;
    default: return OPTORCH_K_RELU_BIAS_BWD;
  }
}

// algorithmic work of one schedule entry: every operand read once, every result written once
void work_of(const optorch_seq_t* h, const SOp& s, double* flops, double* bytes) {
  const FOp& f = h->plan.fops[s.fop];
  const double e = h->plan.esize;
  const double in_px = (double)f.N * f.H * f.W, out_px = (double)f.N * f.P * f.Q;
  const double wts = (double)f.K * f.R * f.S * f.C;
  *flops = 0; *bytes = 0;
  switch (s.kind) {
    case S_CAST_IN: *bytes = in_px * f.C * ((h->x_encoded ? 1 : 4) + e); break;  // an encoded batch: one byte per pixel
    case S_CONV_FWD: *flops = 2 * out_px * wts; *bytes = e * (in_px * f.C + out_px * f.K + wts); break;
    case S_DGRAD:
      *flops = 2 * out_px * wts;
      *bytes = e * (in_px * f.C * (s.in[1] >= 0 ? 2 : 1) + out_px * f.K + wts) + (s.in[2] >= 0 ? e * in_px * f.C / 16 : 0);
      break;
    case S_WGRAD: *flops = 2 * out_px * wts; *bytes = e * (in_px * f.C + out_px * f.K) + 4 * wts; break;
    case S_BN_STATS: *bytes = s.in[1] >= 0 ? 8.0 * f.stat_blocks * f.C : e * out_px * f.C; break;  // fused: only the block sums
    case S_BN_APPLY:
      if (s.out[1] >= 0) *bytes = e * out_px * f.C * (1.0 + (s.out[0] >= 0 ? 1.0 : 0.0) + 0.25);  // z, [a], pooled
      else *bytes = e * out_px * f.C * ((s.in[2] >= 0 ? 3 : 2) + (s.out[2] >= 0 ? 1.0 / 16 : 0));  // + the ReLU bit mask
      break;
    case S_BN_BWD:
      if (s.variant == 1) { *bytes = e * out_px * f.C * (2 * 1.25 + 1); break; }  // twice (z, pooled gradient), dz
      {  // the reduction reads dA, z and the ReLU source; the apply pass reads them again and writes dz (+ the skip gradient)
        const double src = s.in[3] < 0 ? 0.0 : s.variant == 2 ? 1.0 / 16 : 1.0;  // a bit mask is a sixteenth of a tensor
        *bytes = e * out_px * f.C * (2 + src + 3 + src + (s.out[1] >= 0 ? 1 : 0));
      }
      break;
    case S_POOL_FWD: *bytes = e * (in_px + out_px) * f.C; break;
    case S_POOL_BWD: *bytes = e * (2 * in_px + out_px) * f.C; break;
    case S_RELU_BWD: *bytes = e * 3 * out_px * f.K; break;
    case S_BIAS_GRAD: *bytes = e * out_px * f.K; break;
    case S_HEAD_FWD: *bytes = e * in_px * f.C; break;
    case S_HEAD_BWD: *bytes = e * in_px * f.C; break;
  }
}

hipEvent_t next_event(optorch_seq_t* h) {
  if (h->ev_used == h->ev_pool.size()) {
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    h->ev_pool.push_back(e);
  }
  return h->ev_pool[h->ev_used++];
}

hipEvent_t next_event_cb(void* ctx) { return next_event(static_cast<optorch_seq_t*>(ctx)); }

void harvest(optorch_seq_t* h) {
  for (size_t i = 0; i + 1 < h->ev_used; i += 2) {
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, h->ev_pool[i], h->ev_pool[i + 1]) == hipSuccess) {
      h->prof_ms[h->ev_class[i / 2]] += ms;
      if (h->ev_entry[i / 2] >= 0) h->entry_ms[h->ev_entry[i / 2]] += ms;
    }
  }
  h->ev_used = 0;
  h->ev_class.clear();
  h->ev_entry.clear();
}

}  // namespace

extern "C" int optorch_seq_profile_enable(optorch_seq_t* h, int32_t enable) {
  if (!h) return OPTORCH_E_INVALID;
  if (h->bound) (void)hipStreamSynchronize(h->stream);
  h->ev_used = 0; h->ev_class.clear(); h->ev_entry.clear();
  h->entry_ms.assign(h->plan.sched.size(), 0.0);
  h->prof_steps = 0;
  for (int i = 0; i < OPTORCH_N_KERNEL_CLASSES; ++i) {
    h->prof_launches[i] = h->prof_entries[i] = 0;
    h->prof_ms[i] = h->prof_flops[i] = h->prof_bytes[i] = 0;
  }
  h->profiling = enable != 0;
  return OPTORCH_OK;
}

extern "C" int optorch_seq_profile_select(optorch_seq_t* h, uint32_t class_mask) {
  if (!h) return OPTORCH_E_INVALID;
  h->prof_mask = class_mask;
  return OPTORCH_OK;
}

extern "C" int optorch_seq_profile_read(optorch_seq_t* h, int32_t* steps, uint64_t* launches, uint64_t* entries,
                                        double* gpu_ms, double* flops, double* bytes) {
  if (!h) return OPTORCH_E_INVALID;
  if (h->bound) {
    hipError_t e = hipStreamSynchronize(h->stream);
    if (e != hipSuccess) return hip_fail(h, e, "hipStreamSynchronize");
  }
  harvest(h);
  if (steps) *steps = h->prof_steps;
  for (int i = 0; i < OPTORCH_N_KERNEL_CLASSES; ++i) {
    if (launches) launches[i] = h->prof_launches[i];
    if (entries) entries[i] = h->prof_entries[i];
    if (gpu_ms) gpu_ms[i] = h->prof_ms[i];
    if (flops) flops[i] = h->prof_flops[i];
    if (bytes) bytes[i] = h->prof_bytes[i];
  }
  return OPTORCH_OK;
}

extern "C" int optorch_seq_profile_read_entries(optorch_seq_t* h, int32_t capacity, int32_t* n, int32_t* kind, int32_t* unit,
                                                int32_t* phase, double* gpu_ms, double* flops, double* bytes) {
  if (!h || !n) return OPTORCH_E_INVALID;
  if (h->bound) {
    hipError_t e = hipStreamSynchronize(h->stream);
    if (e != hipSuccess) return hip_fail(h, e, "hipStreamSynchronize");
  }
  harvest(h);
  int32_t cnt = 0;
  for (size_t si = 0; si < h->plan.sched.size(); ++si) {
    const SOp& s = h->plan.sched[si];
    if (!s.live) continue;
    if (cnt < capacity) {
      double fl, by;
      work_of(h, s, &fl, &by);
      if (kind) kind[cnt] = class_of(s.kind, h->plan.fops[s.fop]);
      if (unit) unit[cnt] = h->plan.fops[s.fop].unit;
      if (phase) phase[cnt] = s.phase;
      if (gpu_ms) gpu_ms[cnt] = si < h->entry_ms.size() ? h->entry_ms[si] : 0.0;
      if (flops) flops[cnt] = fl * h->prof_steps;
      if (bytes) bytes[cnt] = by * h->prof_steps;
    }
    ++cnt;
  }
  *n = cnt;
  return OPTORCH_OK;
}

// Inference: the forward entries of the schedule (all segments without keeping, then the last segment), with the
// BatchNorm constants taken from the running statistics and the head stopped at the logits.  The arena offsets of
// those entries are valid on their own: the entries run in schedule order and the plan never lets two live tensors
// overlap.  c describes the batch (fp32 or encoded).
static int predict_run(optorch_seq_t* h, const Ctx& c, float* logits_dev) {
  hipStream_t st = h->stream;
  const int dt = h->dt;
  for (const SOp& s : h->plan.sched) {
    if (!s.live || (s.phase != PH_FWD_NOSAVE && s.phase != PH_FWD_LAST)) continue;
    const FOp& f = h->plan.fops[s.fop];
    switch (s.kind) {
      case S_BN_STATS:
        launch_bn_eval_stats(st, (const float*)(h->pbase + h->off_run) + f.rs_off, c.w32(f.gamma_off), c.w32(f.beta_off),
                             h->eps, f.C, (float*)c.at(s.out[0]));
        break;
      case S_CONV_FWD: {  // as in training, without the per-block channel sums
        SOp t = s;
        t.out[2] = -1;
        run_op(c, t);
        break;
      }
      case S_HEAD_FWD: {
        launch_head_logits(st, dt, c.at(s.in[0]), f.N, f.H * f.W, f.C, f.gap, f.feat_dim, f.classes, c.w32(f.w_off),
                           c.w32(f.b_off), (float*)c.at(s.out[0]), (float*)c.at(s.out[1]));
        hipError_t e = hipMemcpyAsync(logits_dev, c.at(s.out[1]), (size_t)f.N * f.classes * 4, hipMemcpyDeviceToDevice, st);
        if (e != hipSuccess) return hip_fail(h, e, "hipMemcpyAsync(logits)");
        break;
      }
      default:
        run_op(c, s);
    }
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return hip_fail(h, e, "kernel launch");
  e = hipStreamSynchronize(st);
  if (e != hipSuccess) return hip_fail(h, e, "hipStreamSynchronize");
  return OPTORCH_OK;
}

extern "C" int optorch_seq_predict(optorch_seq_t* h, const float* x_dev, float* logits_dev) {
  if (!h) return OPTORCH_E_INVALID;
  if (!h->bound || !h->params_set) return set_err(h, OPTORCH_E_ORDER, "predict before bind/set_params");
  if (!x_dev || !logits_dev) return set_err(h, OPTORCH_E_INVALID, "null pointer");
  Ctx c{h, x_dev, nullptr, h->abase};
  return predict_run(h, c, logits_dev);
}

extern "C" int optorch_seq_predict_encoded(optorch_seq_t* h, const uint64_t* a_dev, int32_t z, const float* scale_host,
                                           const float* shift_host, float* logits_dev) {
  if (!h) return OPTORCH_E_INVALID;
  if (!h->bound || !h->params_set) return set_err(h, OPTORCH_E_ORDER, "predict before bind/set_params");
  if (!a_dev || !logits_dev || !scale_host || !shift_host) return set_err(h, OPTORCH_E_INVALID, "null pointer");
  if (z < 1 || z > 16) return set_err(h, OPTORCH_E_INVALID, "images per group must be 1..16");
  if (h->in_channels < 1 || h->in_channels > 16)
    return set_err(h, OPTORCH_E_INVALID, "an encoded batch needs a network input of 1..16 channels");
  Ctx c{h, nullptr, nullptr, h->abase};
  c.xa = a_dev; c.xz = z; c.xscale = scale_host; c.xshift = shift_host;
  return predict_run(h, c, logits_dev);
}

extern "C" int optorch_seq_debug_unit_output(optorch_seq_t* h, const float* x_dev, int32_t unit, float* out_dev,
                                            uint64_t capacity, uint64_t* count, int32_t* shape_nhwc) {
  if (!h) return OPTORCH_E_INVALID;
  if (!h->bound || !h->params_set) return set_err(h, OPTORCH_E_ORDER, "debug_unit_output before bind/set_params");
  const Plan& p = h->plan;
  if (unit < 0 || unit + 1 >= (int32_t)p.units.size())
    return set_err(h, OPTORCH_E_INVALID, "unit index must name a body unit (not the loss head)");
  const int lt = p.unit_out[unit];
  const LTensor& t = p.tensors[lt];
  const uint64_t n = (uint64_t)(t.n * t.h * t.w * t.c);
  if (count) *count = n;
  if (shape_nhwc) { shape_nhwc[0] = (int32_t)t.n; shape_nhwc[1] = (int32_t)t.h; shape_nhwc[2] = (int32_t)t.w; shape_nhwc[3] = (int32_t)t.c; }
  if (!out_dev) return OPTORCH_OK;  // size query
  if (!x_dev) return set_err(h, OPTORCH_E_INVALID, "null input pointer");
  if (capacity < n) return set_err(h, OPTORCH_E_INVALID, "debug_unit_output: buffer too small");
  // the forward entries of the schedule, as a training step runs them, up to the one that writes the unit's output
  Ctx c{h, x_dev, nullptr, h->abase};
  c.touch_running = false;
  hipStream_t st = h->stream;
  bool found = false;
  for (const SOp& s : p.sched) {
    if (!s.live || (s.phase != PH_FWD_NOSAVE && s.phase != PH_FWD_LAST)) continue;
    if (s.kind == S_HEAD_FWD) break;
    run_op(c, s);
    for (int o : s.out)
      if (o >= 0 && p.insts[o].logical == lt) found = true;
    if (found) {
      for (int o : s.out)
        if (o >= 0 && p.insts[o].logical == lt) { launch_cast_out(st, h->dt, c.at(o), out_dev, (int64_t)n); break; }
      break;
    }
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return hip_fail(h, e, "kernel launch");
  e = hipStreamSynchronize(st);
  if (e != hipSuccess) return hip_fail(h, e, "hipStreamSynchronize");
  if (!found) return set_err(h, OPTORCH_E_INVALID, "this plan never writes the unit's output to memory (it is fused into the next unit)");
  return OPTORCH_OK;
}

extern "C" int optorch_seq_running_stats(const optorch_seq_t* h, float* dst, uint64_t capacity, uint64_t* count,
                                         int32_t is_device) {
  if (!h) return OPTORCH_E_INVALID;
  if (count) *count = h->plan.n_running;
  if (!dst) return OPTORCH_OK;  // size query
  if (!h->bound || !h->params_set) return set_err(h, OPTORCH_E_ORDER, "running_stats before bind/set_params");
  if (capacity < h->plan.n_running) return set_err(h, OPTORCH_E_INVALID, "running_stats: buffer too small");
  hipError_t e = hipStreamSynchronize(h->stream);
  if (e == hipSuccess && h->plan.n_running)
    e = hipMemcpy(dst, h->pbase + h->off_run, h->plan.n_running * 4, is_device ? hipMemcpyDeviceToDevice : hipMemcpyDeviceToHost);
  if (e != hipSuccess) return hip_fail(h, e, "hipMemcpy(running statistics)");
  return OPTORCH_OK;
}

// one training step on the batch that c describes
static int step_run(optorch_seq_t* h, const Ctx& c, float lr, float* loss_out, float* grads_dev, uint64_t* peak_saved_bytes,
                    uint64_t* peak_arena_bytes, float* loss_scale_out, int32_t* step_skipped) {
  hipStream_t st = h->stream;
  launch_step_init(st, c.flags(), c.y, h->plan.cfg.batch, h->plan.cfg.num_classes);
  const bool prof = h->profiling;
  if (prof && h->ev_used > (size_t)1 << 16) harvest(h);  // previous steps are complete: each step ends with a sync
  for (size_t si = 0; si < h->plan.sched.size(); ++si) {
    const SOp& s = h->plan.sched[si];
    if (!s.live) continue;
    const bool timed = prof && ((h->prof_mask >> class_of(s.kind, h->plan.fops[s.fop])) & 1u);
    const size_t ev0 = h->ev_used;
    if (timed) g_launch_timer = LaunchTimer{true, next_event_cb, h};  // every launch of the entry carries its own events
    run_op(c, s);
    if (timed) {
      g_launch_timer.on = false;
      const int k = class_of(s.kind, h->plan.fops[s.fop]);
      double fl, by;
      work_of(h, s, &fl, &by);
      const size_t pairs = (h->ev_used - ev0) / 2;
      for (size_t q = 0; q < pairs; ++q) { h->ev_class.push_back(k); h->ev_entry.push_back((int)si); }
      h->prof_launches[k] += pairs;
      h->prof_entries[k] += 1; h->prof_flops[k] += fl; h->prof_bytes[k] += by;
    }
  }
  const int64_t P = (int64_t)h->plan.n_params;
  {
    const bool timed = prof && ((h->prof_mask >> OPTORCH_K_OPTIMIZER) & 1u);
    const size_t ev0 = h->ev_used;
    if (timed) g_launch_timer = LaunchTimer{true, next_event_cb, h};
    launch_optim(st, h->dt, c.w32(0), (float*)(h->pbase + h->off_v), c.g32(0), h->pbase + h->off_h, grads_dev, P, lr,
                 h->momentum, 1.f / h->scale, c.flags());
    if (timed) {
      g_launch_timer.on = false;
      const int k = OPTORCH_K_OPTIMIZER;
      const size_t pairs = (h->ev_used - ev0) / 2;
      for (size_t q = 0; q < pairs; ++q) { h->ev_class.push_back(k); h->ev_entry.push_back(-1); }
      h->prof_launches[k] += pairs; h->prof_entries[k] += 1;
      // read g (check), read g, w [, v], write w [, v] [, 16-bit copy] [, unscaled g]
      h->prof_bytes[k] += (double)P * (4 + 12 + (h->momentum != 0.f ? 8 : 0) + (h->dt != DT_F32 ? 2 : 0) + (grads_dev ? 4 : 0));
    }
    if (prof) h->prof_steps += 1;
  }
  refresh_transposed_weights(h);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return hip_fail(h, e, "kernel launch");
  e = hipMemcpyAsync(h->host_rb, h->pbase + h->off_scal, 128, hipMemcpyDeviceToHost, st);
  if (e != hipSuccess) return hip_fail(h, e, "hipMemcpyAsync(read-back)");
  e = hipStreamSynchronize(st);
  if (e != hipSuccess) return hip_fail(h, e, "hipStreamSynchronize");
  const int* fl = (const int*)((const char*)h->host_rb + 64);
  if (fl[1]) return set_err(h, OPTORCH_E_INVALID, "a label is outside [0, num_classes)");
  const bool skipped = fl[0] != 0;
  if (skipped) {
    if (h->dynamic_scale) h->scale *= h->backoff;
    h->clean = 0;
  } else if (h->dynamic_scale && ++h->clean == h->growth_interval) {
    h->scale *= h->growth;
    h->clean = 0;
  }
  if (loss_out) *loss_out = h->host_rb[0];
  if (peak_saved_bytes) *peak_saved_bytes = h->plan.peak_saved_bytes;
  if (peak_arena_bytes) *peak_arena_bytes = h->plan.arena_bytes;
  if (loss_scale_out) *loss_scale_out = h->scale;
  if (step_skipped) *step_skipped = skipped ? 1 : 0;
  return OPTORCH_OK;
}

extern "C" int optorch_seq_step(optorch_seq_t* h, const float* x_dev, const int32_t* y_dev, float lr, float* loss_out,
                                float* grads_dev, uint64_t* peak_saved_bytes, uint64_t* peak_arena_bytes,
                                float* loss_scale_out, int32_t* step_skipped) {
  if (!h) return OPTORCH_E_INVALID;
  if (!h->bound || !h->params_set) return set_err(h, OPTORCH_E_ORDER, "step before bind/set_params");
  if (!x_dev || !y_dev) return set_err(h, OPTORCH_E_INVALID, "null input pointer");
  if (!std::isfinite(lr)) return set_err(h, OPTORCH_E_INVALID, "learning rate is not finite");
  Ctx c{h, x_dev, y_dev, h->abase};
  h->x_encoded = false;
  return step_run(h, c, lr, loss_out, grads_dev, peak_saved_bytes, peak_arena_bytes, loss_scale_out, step_skipped);
}

extern "C" int optorch_seq_step_encoded(optorch_seq_t* h, const uint64_t* a_dev, int32_t z, const float* scale_host,
                                        const float* shift_host, const int32_t* y_dev, float lr, float* loss_out,
                                        float* grads_dev, uint64_t* peak_saved_bytes, uint64_t* peak_arena_bytes,
                                        float* loss_scale_out, int32_t* step_skipped) {
  if (!h) return OPTORCH_E_INVALID;
  if (!h->bound || !h->params_set) return set_err(h, OPTORCH_E_ORDER, "step before bind/set_params");
  if (!a_dev || !y_dev || !scale_host || !shift_host) return set_err(h, OPTORCH_E_INVALID, "null input pointer");
  if (z < 1 || z > 16) return set_err(h, OPTORCH_E_INVALID, "images per group must be 1..16");
  if (h->in_channels < 1 || h->in_channels > 16)
    return set_err(h, OPTORCH_E_INVALID, "an encoded batch needs a network input of 1..16 channels");
  if (!std::isfinite(lr)) return set_err(h, OPTORCH_E_INVALID, "learning rate is not finite");
  Ctx c{h, nullptr, y_dev, h->abase};
  c.xa = a_dev; c.xz = z; c.xscale = scale_host; c.xshift = shift_host;
  h->x_encoded = true;
  return step_run(h, c, lr, loss_out, grads_dev, peak_saved_bytes, peak_arena_bytes, loss_scale_out, step_skipped);
}

extern "C" int optorch_seq_step_static(optorch_seq_t* h, const float* x_dev, const int32_t* y_dev, float lr, float* loss_out,
                                       float* grads_dev, uint64_t* peak_saved_bytes, uint64_t* peak_arena_bytes,
                                       float* loss_scale_out, int32_t* step_skipped) {
  if (!h) return OPTORCH_E_INVALID;
  if (!h->bound || !h->params_set) return set_err(h, OPTORCH_E_ORDER, "step before bind/set_params");
  if (!x_dev || !y_dev) return set_err(h, OPTORCH_E_INVALID, "null input pointer");
  if (!std::isfinite(lr)) return set_err(h, OPTORCH_E_INVALID, "learning rate is not finite");
  if (h->profiling) return set_err(h, OPTORCH_E_ORDER, "optorch_seq_step_static does not time launches: disable profiling");
  if (h->plan.arena_bytes > (uint64_t)OPTORCH_STATIC_ARENA_BYTES)
    return set_err(h, OPTORCH_E_BUDGET, "planned activation arena of " + std::to_string(h->plan.arena_bytes) +
                                            " bytes exceeds the static arena of " +
                                            std::to_string((uint64_t)OPTORCH_STATIC_ARENA_BYTES) + " bytes");
  void* arena = nullptr;
  uint64_t bytes = 0;
  hipError_t e = static_arena(&arena, &bytes);
  if (e != hipSuccess) return hip_fail(h, e, "hipGetSymbolAddress(static arena)");
  Ctx c{h, x_dev, y_dev, (char*)arena};
  h->x_encoded = false;
  return step_run(h, c, lr, loss_out, grads_dev, peak_saved_bytes, peak_arena_bytes, loss_scale_out, step_skipped);
}

extern "C" const char* optorch_seq_last_error(const optorch_seq_t* h) { return h ? h->err.c_str() : g_create_error.c_str(); }

extern "C" void optorch_seq_destroy(optorch_seq_t* h) {
  if (!h) return;
  if (h->host_rb) (void)hipHostFree(h->host_rb);
  for (hipEvent_t e : h->ev_pool) (void)hipEventDestroy(e);
  delete h;
}
