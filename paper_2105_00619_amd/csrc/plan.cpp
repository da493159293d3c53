// Host-side planner; see plan.h.
#include "plan.h"

#include <algorithm>
#include <cstdio>
#include <map>

namespace oseq {

namespace {

struct ConvParams { int64_t w = -1, b = -1, gamma = -1, beta = -1, rs = -1; };

struct Builder {
  Plan& p;
  int N;
  explicit Builder(Plan& pl) : p(pl), N(pl.cfg.batch) {}

  bool fail(const std::string& m) { p.error = m; return false; }

  int new_tensor(int64_t n, int64_t h, int64_t w, int64_t c, int esize, int unit) {
    LTensor t;
    t.n = n; t.h = h; t.w = w; t.c = c; t.esize = esize; t.unit = unit;
    t.bytes = (uint64_t)n * h * w * c * esize;
    p.tensors.push_back(t);
    return (int)p.tensors.size() - 1;
  }

  ConvParams alloc_conv_params(int cin, int cout, int k, int bn, int bias) {
    ConvParams q;
    q.w = (int64_t)p.n_params; p.n_params += (uint64_t)cout * k * k * cin;
    if (bias) { q.b = (int64_t)p.n_params; p.n_params += cout; }
    if (bn) {
      q.gamma = (int64_t)p.n_params; p.n_params += cout;
      q.beta = (int64_t)p.n_params; p.n_params += cout;
      q.rs = (int64_t)p.n_running; p.n_running += 2 * (uint64_t)cout;
    }
    return q;
  }

  // conv [+bias] [+BN [+skip]] [+ReLU]; appends the forward operations, returns the output tensor
  int add_cbr(int unit, int x, const ConvParams& q, int cout, int k, int stride, int pad, int bn,
              int relu, int bias, int skip) {
    const LTensor tx = p.tensors[x];
    FOp f;
    f.kind = F_CONV; f.unit = unit; f.x = x;
    f.N = (int)tx.n; f.H = (int)tx.h; f.W = (int)tx.w; f.C = (int)tx.c; f.K = cout; f.R = k; f.S = k;
    f.stride = stride; f.pad = pad;
    f.P = (f.H + 2 * pad - k) / stride + 1;
    f.Q = (f.W + 2 * pad - k) / stride + 1;
    f.has_bias = bias; f.has_bn = bn; f.relu = bn ? 0 : relu;
    f.w_off = q.w; f.b_off = q.b;
    const int64_t pixels = (int64_t)f.N * f.P * f.Q;
    const int64_t outputs = (int64_t)f.K * f.R * f.S * f.C;
    int64_t splits = (262144 + outputs - 1) / outputs;
    splits = std::min<int64_t>(splits, std::max<int64_t>(1, pixels / 32));
    f.wgrad_splits = (int)std::max<int64_t>(1, std::min<int64_t>(splits, 256));
    f.red_blocks = (int)std::max<int64_t>(1, std::min<int64_t>(pixels / 32, 512));
    int z = new_tensor(f.N, f.P, f.Q, cout, p.esize, unit);
    f.out = z;
    p.fops.push_back(f);
    if (!bn) return z;

    FOp s;
    s.kind = F_BN_STATS; s.unit = unit; s.x = z;
    s.N = f.N; s.H = f.P; s.W = f.Q; s.C = cout; s.K = cout; s.P = f.P; s.Q = f.Q;
    s.gamma_off = q.gamma; s.beta_off = q.beta; s.rs_off = q.rs;
    s.red_blocks = (int)std::max<int64_t>(1, std::min<int64_t>(pixels / 32, 512));
    s.stats = new_tensor(1, 1, 4, cout, 4, unit);  // mean, rstd, scale, shift
    s.out = s.stats;
    p.fops.push_back(s);

    FOp a = s;
    a.kind = F_BN_APPLY; a.skip = skip; a.relu = relu;
    a.out = new_tensor(f.N, f.P, f.Q, cout, p.esize, unit);
    // The ReLU behind a skip connection cannot be redone from z alone; backward needs its decisions.  They are kept as
    // one bit per element (one byte per group of 16 / esize channels), a sixteenth of the bytes of the output that
    // backward would otherwise read twice.
    const int vgroup = 16 / p.esize;
    if (skip >= 0 && relu && cout % vgroup == 0) {
      a.mask = new_tensor(f.N, f.P, f.Q, cout / vgroup, 1, unit);
      p.tensors[a.mask].needs_grad = false;
    }
    p.fops.push_back(a);
    return a.out;
  }

  bool run() {
    const optorch_seq_config_t& c = p.cfg;
    p.esize = c.precision == OPTORCH_FP32 ? 4 : 2;
    if (p.units.empty()) return fail("empty unit list");
    int cur = new_tensor(N, c.height, c.width, c.channels, p.esize, -1);
    p.tensors[cur].needs_grad = false;
    {
      FOp f; f.kind = F_CAST_IN; f.unit = -1; f.out = cur;
      f.N = N; f.H = c.height; f.W = c.width; f.C = c.channels;
      p.fops.push_back(f);
    }
    const int nu = (int)p.units.size();
    p.unit_first_fop.assign(nu, 0); p.unit_last_fop.assign(nu, 0);
    p.unit_in.assign(nu, -1); p.unit_out.assign(nu, -1);
    for (int ui = 0; ui < nu; ++ui) {
      const optorch_unit_t& u = p.units[ui];
      const LTensor tx = p.tensors[cur];
      p.unit_first_fop[ui] = (int)p.fops.size();
      p.unit_in[ui] = cur;
      char where[64]; snprintf(where, sizeof where, "unit %d: ", ui);
      const bool is_head = u.kind == OPTORCH_GAP_LINEAR_CE || u.kind == OPTORCH_FLATTEN_LINEAR_CE;
      if (is_head != (ui == nu - 1)) return fail(std::string(where) + "exactly the last unit must be a loss head");
      switch (u.kind) {
        case OPTORCH_CONV: {
          if (u.cin != tx.c) return fail(std::string(where) + "cin does not match the incoming channel count");
          if (!(u.ksize == 1 || u.ksize == 3) || !(u.stride == 1 || u.stride == 2) || u.cout < 1 || u.pad < 0 ||
              u.pad > u.ksize / 2)
            return fail(std::string(where) + "unsupported convolution geometry (ksize 1|3, stride 1|2, pad <= ksize/2)");
          if (tx.h + 2 * u.pad < u.ksize || tx.w + 2 * u.pad < u.ksize) return fail(std::string(where) + "input smaller than the filter");
          ConvParams q = alloc_conv_params(u.cin, u.cout, u.ksize, u.has_bn, u.has_bias);
          cur = add_cbr(ui, cur, q, u.cout, u.ksize, u.stride, u.pad, u.has_bn != 0, u.has_relu != 0, u.has_bias != 0, -1);
          break;
        }
        case OPTORCH_MAXPOOL2: {
          if (tx.h < 2 || tx.w < 2) return fail(std::string(where) + "max-pool input smaller than 2x2");
          FOp f; f.kind = F_POOL; f.unit = ui; f.x = cur;
          f.N = N; f.H = (int)tx.h; f.W = (int)tx.w; f.C = (int)tx.c; f.K = f.C; f.P = f.H / 2; f.Q = f.W / 2;
          f.out = new_tensor(N, f.P, f.Q, f.C, p.esize, ui);
          p.fops.push_back(f);
          cur = f.out;
          break;
        }
        case OPTORCH_BASIC_BLOCK:
        case OPTORCH_BOTTLENECK: {
          if (u.cin != tx.c) return fail(std::string(where) + "cin does not match the incoming channel count");
          if (!(u.stride == 1 || u.stride == 2) || u.cout < 1) return fail(std::string(where) + "unsupported block geometry");
          const bool bott = u.kind == OPTORCH_BOTTLENECK;
          if (bott && (u.cout % 4 != 0)) return fail(std::string(where) + "bottleneck cout must be a multiple of 4");
          const bool proj = (u.cin != u.cout) || (u.stride != 1);
          const int mid = bott ? u.cout / 4 : u.cout;
          ConvParams q1, q2, q3, qs;
          if (bott) {
            q1 = alloc_conv_params(u.cin, mid, 1, 1, 0);
            q2 = alloc_conv_params(mid, mid, 3, 1, 0);
            q3 = alloc_conv_params(mid, u.cout, 1, 1, 0);
          } else {
            q1 = alloc_conv_params(u.cin, u.cout, 3, 1, 0);
            q2 = alloc_conv_params(u.cout, u.cout, 3, 1, 0);
          }
          if (proj) qs = alloc_conv_params(u.cin, u.cout, 1, 1, 0);
          const int x = cur;
          int a;
          if (bott) {
            a = add_cbr(ui, x, q1, mid, 1, 1, 0, 1, 1, 0, -1);
            a = add_cbr(ui, a, q2, mid, 3, u.stride, 1, 1, 1, 0, -1);
          } else {
            a = add_cbr(ui, x, q1, u.cout, 3, u.stride, 1, 1, 1, 0, -1);
          }
          int skip = x;
          if (proj) skip = add_cbr(ui, x, qs, u.cout, 1, u.stride, 0, 1, 0, 0, -1);
          if (bott) cur = add_cbr(ui, a, q3, u.cout, 1, 1, 0, 1, 1, 0, skip);
          else      cur = add_cbr(ui, a, q2, u.cout, 3, 1, 1, 1, 1, 0, skip);
          break;
        }
        case OPTORCH_GAP_LINEAR_CE:
        case OPTORCH_FLATTEN_LINEAR_CE: {
          if (u.cin != tx.c) return fail(std::string(where) + "cin does not match the incoming channel count");
          if (u.cout != c.num_classes) return fail(std::string(where) + "cout must equal num_classes");
          FOp f; f.kind = F_HEAD; f.unit = ui; f.x = cur;
          f.N = N; f.H = (int)tx.h; f.W = (int)tx.w; f.C = (int)tx.c;
          f.gap = u.kind == OPTORCH_GAP_LINEAR_CE;
          f.feat_dim = f.gap ? f.C : f.H * f.W * f.C;
          f.classes = u.cout; f.has_bias = 1;
          f.w_off = (int64_t)p.n_params; p.n_params += (uint64_t)f.classes * f.feat_dim;
          f.b_off = (int64_t)p.n_params; p.n_params += f.classes;
          f.aux[0] = new_tensor(N, 1, 1, f.feat_dim, 4, ui);
          f.aux[1] = new_tensor(N, 1, 1, f.classes, 4, ui);
          f.aux[2] = new_tensor(N, 1, 1, f.classes, 4, ui);
          f.out = new_tensor(N, 1, 1, 1, 4, ui);
          p.fops.push_back(f);
          cur = f.out;
          break;
        }
        default:
          return fail(std::string(where) + "unknown unit kind");
      }
      p.unit_last_fop[ui] = (int)p.fops.size();
      p.unit_out[ui] = cur;
    }
    return true;
  }
};

// ---------------------------------------------------------------- arena -----
struct FreeList {
  std::map<uint64_t, uint64_t> free_;  // offset -> size
  uint64_t end_ = 0;                    // current top of the arena
  uint64_t high_ = 0;

  uint64_t alloc(uint64_t bytes) {
    bytes = align_up(std::max<uint64_t>(bytes, 1));
    auto best = free_.end();
    for (auto it = free_.begin(); it != free_.end(); ++it)
      if (it->second >= bytes && (best == free_.end() || it->second < best->second)) best = it;
    if (best != free_.end()) {
      uint64_t off = best->first, sz = best->second;
      free_.erase(best);
      if (sz > bytes) free_[off + bytes] = sz - bytes;
      return off;
    }
    // grow: extend a free block that touches the top, if any
    uint64_t off = end_;
    if (!free_.empty()) {
      auto last = std::prev(free_.end());
      if (last->first + last->second == end_) { off = last->first; free_.erase(last); }
    }
    end_ = off + bytes;
    high_ = std::max(high_, end_);
    return off;
  }
  void release(uint64_t off, uint64_t bytes) {
    bytes = align_up(std::max<uint64_t>(bytes, 1));
    auto it = free_.emplace(off, bytes).first;
    auto nx = std::next(it);
    if (nx != free_.end() && it->first + it->second == nx->first) { it->second += nx->second; free_.erase(nx); }
    if (it != free_.begin()) {
      auto pv = std::prev(it);
      if (pv->first + pv->second == it->first) { pv->second += it->second; free_.erase(it); it = pv; }
    }
    if (it->first + it->second == end_) { end_ = it->first; free_.erase(it); }
  }
};

bool is_fwd_kind(SKind k) { return k <= S_HEAD_FWD; }

bool has_side_effect(SKind k) {
  // writes parameter gradients, the loss, or BN running statistics
  return k == S_HEAD_FWD || k == S_HEAD_BWD || k == S_BN_BWD || k == S_BIAS_GRAD || k == S_WGRAD || k == S_BN_STATS;
}

struct Scheduler {
  Plan& p;
  std::vector<int> cur, grad;  // [LTensor] -> Inst id
  std::vector<int> stat_ws;    // [LTensor of a conv output] -> Inst id of the channel sums its forward kernel wrote
  std::vector<int> bn_apply_of;  // [LTensor] -> the F_BN_APPLY operation that produces it, or -1
  std::vector<char> rebuilt;     // [LTensor] backward has already rebuilt it (storage mode 1)
  std::vector<int> readers;      // [LTensor] -> number of forward operations that read it
  std::vector<int> via_pool;     // [LTensor] -> Inst id of the gradient of the max-pool output behind it, when the
                                 //              pool's backward is left to the BatchNorm backward in front of it
  std::vector<int> gmask;        // [LTensor] -> Inst id of a ReLU bit mask that grad[t] still has to be multiplied by
                                 //              (the gradient through a skip connection is not written out: its
                                 //              reader applies the mask to the block output's gradient itself), or -1
  explicit Scheduler(Plan& pl)
      : p(pl), cur(pl.tensors.size(), -1), grad(pl.tensors.size(), -1), stat_ws(pl.tensors.size(), -1),
        bn_apply_of(pl.tensors.size(), -1), rebuilt(pl.tensors.size(), 0), readers(pl.tensors.size(), 0),
        via_pool(pl.tensors.size(), -1), gmask(pl.tensors.size(), -1) {
    for (size_t fi = 0; fi < pl.fops.size(); ++fi) {
      const FOp& f = pl.fops[fi];
      if (f.kind == F_BN_APPLY) bn_apply_of[f.out] = (int)fi;
      if (f.x >= 0) ++readers[f.x];
      if (f.skip >= 0) ++readers[f.skip];
    }
  }

  // Is forward operation fi a 2x2 max-pool whose backward the BatchNorm backward in front of it does as well?  The
  // activation between them must be read by nothing else; the rule looks at the network only (never at the segments),
  // so the sums of that BatchNorm backward are added in the same order for every k.
  bool pool_bwd_fused(int fi) const {
    if (fi < 1) return false;
    const FOp& pool = p.fops[fi];
    const FOp& ap = p.fops[fi - 1];
    if (pool.kind != F_POOL || ap.kind != F_BN_APPLY || pool.x != ap.out || ap.skip >= 0) return false;
    return ap.P % 2 == 0 && ap.Q % 2 == 0 && readers[ap.out] == 1 && p.tensors[ap.out].needs_grad;
  }

  int new_inst(int logical, uint64_t bytes, bool fwd_value) {
    Inst i; i.logical = logical; i.bytes = bytes; i.fwd_value = fwd_value;
    p.insts.push_back(i);
    return (int)p.insts.size() - 1;
  }
  int value_inst(int t) { return cur[t] = new_inst(t, p.tensors[t].bytes, true); }
  int grad_inst(int t) { return new_inst(t, p.tensors[t].bytes, false); }

  SOp& push(SKind k, int fop, int phase, int seg) {
    SOp s; s.kind = k; s.fop = fop; s.phase = phase; s.seg = seg;
    p.sched.push_back(s);
    return p.sched.back();
  }

  // Is forward operation fi a 2x2 max-pool that the BatchNorm apply right in front of it computes as well?  Both must
  // lie in segment `seg` (a pool that opens a segment is replayed from the segment's kept input), the apply must add
  // no skip connection, and the map must have even sides.
  bool pool_fused(int fi, int seg) const {
    if (fi < 1 || fi >= (int)p.fops.size()) return false;
    const FOp& pool = p.fops[fi];
    const FOp& ap = p.fops[fi - 1];
    if (pool.kind != F_POOL || ap.kind != F_BN_APPLY || pool.x != ap.out || ap.skip >= 0) return false;
    if (ap.P % 2 != 0 || ap.Q % 2 != 0) return false;
    return ap.unit >= p.seg_begin[seg] && pool.unit < p.seg_begin[seg + 1];
  }

  void emit_fop_forward(int fi, int phase, int seg) {
    const FOp& f = p.fops[fi];
    switch (f.kind) {
      case F_CAST_IN: { SOp& s = push(S_CAST_IN, fi, phase, seg); s.out[0] = value_inst(f.out); break; }
      case F_CONV: {
        SOp& s = push(S_CONV_FWD, fi, phase, seg);
        s.in[0] = cur[f.x];
        if (f.fold_src >= 0) { s.in[0] = cur[p.fops[f.fold_src].x]; s.in[1] = cur[p.fops[f.fold_src].stats]; }
        s.out[0] = value_inst(f.out);
        if (f.fwd_splits > 1) s.out[1] = new_inst(-1, (uint64_t)f.fwd_splits * f.N * f.P * f.Q * f.K * 4, false);
        if (f.stat_blocks > 0 && phase != PH_REPLAY) {  // per-block channel sums for the BatchNorm that follows
          s.out[2] = new_inst(-1, (uint64_t)(f.stat_blocks + f.stat_fold) * 2 * f.K * 4, false);
          stat_ws[f.out] = s.out[2];
        }
        break;
      }
      case F_BN_STATS: {
        if (phase == PH_REPLAY) break;  // the statistics of the first forward pass are kept and reused
        SOp& s = push(S_BN_STATS, fi, phase, seg);
        s.in[0] = cur[f.x]; s.out[0] = value_inst(f.stats);
        if (f.stat_blocks > 0) s.in[1] = stat_ws[f.x];  // sums come from the convolution: only the finishing kernel runs
        else s.out[1] = new_inst(-1, (uint64_t)f.red_blocks * 2 * f.C * 4, false);
        break;
      }
      case F_BN_APPLY: {
        if (f.fold) break;  // done by the convolution that reads it
        SOp& s = push(S_BN_APPLY, fi, phase, seg);
        s.in[0] = cur[f.x]; s.in[1] = cur[f.stats]; s.in[2] = f.skip >= 0 ? cur[f.skip] : -1;
        s.out[0] = value_inst(f.out);
        if (pool_fused(fi + 1, seg)) s.out[1] = value_inst(p.fops[fi + 1].out);  // the same kernel also pools
        if (f.mask >= 0) s.out[2] = value_inst(f.mask);
        break;
      }
      case F_POOL: {
        if (pool_fused(fi, seg)) break;  // done by the BatchNorm apply in front of it
        SOp& s = push(S_POOL_FWD, fi, phase, seg); s.in[0] = cur[f.x]; s.out[0] = value_inst(f.out);
        break;
      }
      case F_HEAD: {
        SOp& s = push(S_HEAD_FWD, fi, phase, seg);
        s.in[0] = cur[f.x];
        s.out[0] = value_inst(f.aux[0]); s.out[1] = value_inst(f.aux[1]);
        s.out[2] = value_inst(f.aux[2]); s.out[3] = value_inst(f.out);
        break;
      }
    }
  }

  // The instance of forward tensor t that a backward operation of segment `seg` reads.  Storage mode 1: an
  // activation A = ReLU(BN(Z)) without a skip connection, produced inside this segment, is not kept from the forward
  // pass; the first backward operation that needs it has it rebuilt from Z and the kept statistics by the same
  // elementwise kernel (hence the same bits), as a transient of the backward pass.
  int backward_input(int t, int seg) {
    const int fa = bn_apply_of[t];
    if (p.cfg.storage_mode != 1 || fa < 0 || rebuilt[t]) return cur[t];
    const FOp& f = p.fops[fa];
    if (f.skip >= 0 || f.unit < p.seg_begin[seg] || f.unit >= p.seg_begin[seg + 1]) return cur[t];
    SOp& s = push(S_BN_APPLY, fa, PH_BWD, seg);
    s.in[0] = cur[f.x]; s.in[1] = cur[f.stats];
    s.out[0] = cur[t] = new_inst(t, p.tensors[t].bytes, false);
    rebuilt[t] = 1;
    return cur[t];
  }

  // May the reader of the gradient through operation fi's skip connection take it as (gradient of the block output,
  // ReLU bit mask) instead of a tensor of its own?  A BatchNorm backward (projection shortcut) always can; a
  // convolution's data gradient can where it runs on the matrix cores (their shared epilogue applies the mask).
  bool masked_skip_grad_ok(int fi) const {
    const FOp& f = p.fops[fi];
    if (f.mask < 0 || f.skip < 0) return false;
    if (bn_apply_of[f.skip] >= 0 && p.fops[bn_apply_of[f.skip]].unit == f.unit) return true;
    for (int j = p.unit_first_fop[f.unit]; j < p.unit_last_fop[f.unit]; ++j)
      if (p.fops[j].kind == F_CONV && p.fops[j].x == f.skip) return p.fops[j].dgrad_algo == ALGO_MFMA;
    return false;
  }

  bool emit_fop_backward(int fi, int seg) {
    const FOp& f = p.fops[fi];
    switch (f.kind) {
      case F_CAST_IN: case F_BN_STATS: return true;
      case F_HEAD: {
        SOp& s = push(S_HEAD_BWD, fi, PH_BWD, seg);
        s.in[0] = cur[f.aux[0]]; s.in[1] = cur[f.aux[2]];
        if (p.tensors[f.x].needs_grad) { s.out[0] = grad_inst(f.x); grad[f.x] = s.out[0]; }
        s.out[1] = new_inst(-1, (uint64_t)f.N * f.feat_dim * 4, false);
        return true;
      }
      case F_BN_APPLY: {
        int gin = grad[f.out], variant = 0;
        if (gin < 0 && via_pool[f.out] >= 0) { gin = via_pool[f.out]; variant = 1; }  // through the pool behind it
        if (gin < 0) { p.error = "internal: BN output has no gradient"; return false; }
        if (f.skip >= 0 && !f.relu) { p.error = "skip connection without ReLU is not supported"; return false; }
        const int gin_mask = gmask[f.out];  // the incoming gradient still wants a mask (projection shortcut's BatchNorm)
        SOp& s = push(S_BN_BWD, fi, PH_BWD, seg);
        s.variant = variant;
        s.in[0] = gin; s.in[1] = cur[f.x]; s.in[2] = cur[f.stats];
        s.in[3] = (f.skip >= 0) ? cur[f.out] : -1;
        if (gin_mask >= 0) {
          if (f.skip >= 0 || variant != 0) { p.error = "internal: masked gradient into a BatchNorm with a skip connection"; return false; }
          s.in[3] = gin_mask; s.variant = 2;
        } else if (f.mask >= 0) {
          s.in[3] = cur[f.mask]; s.variant = 2;
        }
        s.out[0] = grad_inst(f.x); grad[f.x] = s.out[0]; gmask[f.x] = -1;
        if (f.skip >= 0 && p.tensors[f.skip].needs_grad) {
          if (grad[f.skip] >= 0) { p.error = "internal: skip gradient must be the first contribution"; return false; }
          if (masked_skip_grad_ok(fi)) { grad[f.skip] = gin; gmask[f.skip] = cur[f.mask]; }  // nothing written
          else { s.out[1] = grad_inst(f.skip); grad[f.skip] = s.out[1]; gmask[f.skip] = -1; }
        }
        s.out[2] = new_inst(-1, ((uint64_t)f.red_blocks * 2 + 2) * f.C * 4, false);
        return true;
      }
      case F_CONV: {
        int g = grad[f.out];
        if (g < 0) { p.error = "internal: conv output has no gradient"; return false; }
        if (!f.has_bn && f.relu) {
          SOp& s = push(S_RELU_BWD, fi, PH_BWD, seg);
          s.in[0] = g; s.in[1] = cur[f.out];
          s.out[0] = grad_inst(f.out); g = s.out[0];
        }
        if (f.has_bias) {
          SOp& s = push(S_BIAS_GRAD, fi, PH_BWD, seg);
          s.in[0] = g;
          s.out[0] = new_inst(-1, (uint64_t)f.red_blocks * 2 * f.K * 4, false);
        }
        {
          const int xin = f.fold_src >= 0 ? cur[p.fops[f.fold_src].x] : backward_input(f.x, seg);
          SOp& s = push(S_WGRAD, fi, PH_BWD, seg);
          s.in[0] = xin; s.in[1] = g;
          if (f.fold_src >= 0) s.in[2] = cur[p.fops[f.fold_src].stats];
          if (f.wgrad_splits > 1)
            s.out[0] = new_inst(-1, (uint64_t)f.wgrad_splits * f.K * f.R * f.S * f.C * 4, false);
        }
        if (p.tensors[f.x].needs_grad) {
          SOp& s = push(S_DGRAD, fi, PH_BWD, seg);
          s.in[0] = g; s.in[1] = grad[f.x]; s.in[2] = grad[f.x] >= 0 ? gmask[f.x] : -1;
          s.out[0] = grad_inst(f.x); grad[f.x] = s.out[0]; gmask[f.x] = -1;
          if (f.dgrad_splits > 1) s.out[1] = new_inst(-1, (uint64_t)f.dgrad_splits * f.N * f.H * f.W * f.C * 4, false);
        }
        return true;
      }
      case F_POOL: {
        if (grad[f.out] < 0) { p.error = "internal: pool output has no gradient"; return false; }
        if (!p.tensors[f.x].needs_grad) return true;
        if (grad[f.x] >= 0) { p.error = "internal: pool input already has a gradient"; return false; }
        if (pool_bwd_fused(fi)) { via_pool[f.x] = grad[f.out]; return true; }
        const int xin = backward_input(f.x, seg);
        SOp& s = push(S_POOL_BWD, fi, PH_BWD, seg);
        s.in[0] = xin; s.in[1] = grad[f.out];
        s.out[0] = grad_inst(f.x); grad[f.x] = s.out[0];
        return true;
      }
    }
    return true;
  }

  bool run() {
    const int k = (int)p.seg_begin.size() - 1;
    p.insts.clear(); p.sched.clear();
    emit_fop_forward(0, k == 1 ? PH_FWD_LAST : PH_FWD_NOSAVE, 0);
    auto forward_seg = [&](int j, int phase) {
      for (int u = p.seg_begin[j]; u < p.seg_begin[j + 1]; ++u)
        for (int fi = p.unit_first_fop[u]; fi < p.unit_last_fop[u]; ++fi) emit_fop_forward(fi, phase, j);
    };
    for (int j = 0; j < k - 1; ++j) forward_seg(j, PH_FWD_NOSAVE);
    forward_seg(k - 1, PH_FWD_LAST);
    for (int j = k - 1; j >= 0; --j) {
      if (j < k - 1) forward_seg(j, PH_REPLAY);
      for (int u = p.seg_begin[j + 1] - 1; u >= p.seg_begin[j]; --u)
        for (int fi = p.unit_last_fop[u] - 1; fi >= p.unit_first_fop[u]; --fi)
          if (!emit_fop_backward(fi, j)) return false;
    }
    return true;
  }
};

}  // namespace

int launches_of(const SOp& op, const FOp& f) {
  switch (op.kind) {
    case S_BN_STATS: return f.stat_blocks > 0 ? (f.stat_fold > 0 ? 2 : 1) : 2;
    case S_HEAD_FWD: return 4;
    case S_HEAD_BWD: return op.out[0] >= 0 ? 4 : 2;
    case S_BN_BWD: return 3;
    case S_BIAS_GRAD: return 2;
    case S_WGRAD: return f.wgrad_splits > 1 ? 2 : 1;
    case S_CONV_FWD: return f.fwd_splits > 1 ? 2 : 1;
    case S_DGRAD: return f.dgrad_splits > 1 ? 2 : 1;
    default: return 1;
  }
}

bool build_graph(Plan& p) {
  p.tensors.clear(); p.fops.clear(); p.n_params = 0; p.n_running = 0;
  const optorch_seq_config_t& c = p.cfg;
  if (c.batch < 1 || c.height < 1 || c.width < 1 || c.channels < 1 || c.num_classes < 2) {
    p.error = "batch, height, width, channels must be >= 1 and num_classes >= 2";
    return false;
  }
  if (c.precision < 0 || c.precision > 2) { p.error = "precision must be 0 (fp32), 1 (bf16) or 2 (fp16)"; return false; }
  if (c.storage_mode < 0 || c.storage_mode > 2) { p.error = "storage_mode must be 0, 1 or 2"; return false; }
  if ((int64_t)c.batch * c.height * c.width * 2048 > (int64_t)1 << 40) { p.error = "batch too large"; return false; }
  Builder b(p);
  return b.run();
}

bool build_schedule(Plan& p) {
  Scheduler s(p);
  if (!s.run()) return false;
  const int n = (int)p.sched.size();
  // dead-operation elimination (a replayed operation whose result nobody reads is not run)
  std::vector<int> uses(p.insts.size(), 0);
  for (int i = n - 1; i >= 0; --i) {
    SOp& op = p.sched[i];
    bool live = has_side_effect(op.kind);
    for (int o : op.out) if (o >= 0 && uses[o] > 0) live = true;
    op.live = live;
    if (live && op.kind == S_BN_APPLY && op.out[1] >= 0) {  // apply + pool: an output nobody reads is not written
      if (uses[op.out[0]] == 0) op.out[0] = -1;
      else if (uses[op.out[1]] == 0) op.out[1] = -1;
    }
    if (live && op.kind == S_BN_APPLY && op.out[2] >= 0 && uses[op.out[2]] == 0) op.out[2] = -1;  // the mask likewise
    if (live) for (int x : op.in) if (x >= 0) ++uses[x];
  }
  // lifetimes
  for (Inst& t : p.insts) { t.def_op = -1; t.last_use = -1; t.held = false; t.allocated = false; }
  for (int i = 0; i < n; ++i) {
    const SOp& op = p.sched[i];
    if (!op.live) continue;
    for (int o : op.out) if (o >= 0) { p.insts[o].def_op = i; p.insts[o].last_use = std::max(p.insts[o].last_use, i); }
    for (int x : op.in) if (x >= 0) {
      Inst& t = p.insts[x];
      if (t.def_op < 0) { p.error = "internal: operation reads a tensor that was never produced"; return false; }
      t.last_use = std::max(t.last_use, i);
      const SOp& d = p.sched[t.def_op];
      if (t.fwd_value && (op.phase == PH_BWD || op.phase != d.phase || op.seg != d.seg)) t.held = true;
    }
  }
  // arena offsets + peak figures, by walking the schedule
  std::vector<std::vector<int>> dies(n);
  for (size_t t = 0; t < p.insts.size(); ++t)
    if (p.insts[t].def_op >= 0) dies[p.insts[t].last_use].push_back((int)t);
  FreeList fl;
  uint64_t live_b = 0, held_b = 0;
  p.peak_saved_bytes = p.peak_live_bytes = 0;
  p.n_launches = p.n_replay_launches = 0;
  for (int i = 0; i < n; ++i) {
    const SOp& op = p.sched[i];
    if (!op.live) continue;
    int nl = launches_of(op, p.fops[op.fop]);
    p.n_launches += nl;
    if (op.phase == PH_REPLAY) p.n_replay_launches += nl;
    for (int o : op.out) if (o >= 0) {
      Inst& t = p.insts[o];
      t.offset = fl.alloc(t.bytes); t.allocated = true;
      live_b += t.bytes;
      if (t.held) held_b += t.bytes;
    }
    p.peak_live_bytes = std::max(p.peak_live_bytes, live_b);
    p.peak_saved_bytes = std::max(p.peak_saved_bytes, held_b);
    for (int t : dies[i]) {
      Inst& x = p.insts[t];
      fl.release(x.offset, x.bytes);
      live_b -= x.bytes;
      if (x.held) held_b -= x.bytes;
    }
  }
  p.arena_bytes = fl.high_;
  return true;
}

// Per-unit byte model of what a segment holds for its backward pass, read off a k = 1 schedule.  A tensor kept for
// backward counts for the unit that made it, except a unit's output: that is kept as the input of the next unit (whose
// backward reads it), so inside a segment it counts for every unit but the last, and for the last one only where the
// unit's own backward reads it.  The first unit's input is the segment's checkpoint and is counted separately.
struct SegModel {
  std::vector<uint64_t> own_pre, out_pre, out_self, ck;
  explicit SegModel(const Plan& all) {
    const int nu = (int)all.units.size();
    std::vector<uint64_t> own(nu, 0), outb(nu, 0);
    std::vector<char> self(nu, 0);
    for (const Inst& t : all.insts) {
      if (!t.held || t.logical < 0) continue;
      const int u = all.tensors[t.logical].unit;
      if (u < 0) continue;
      if (t.logical == all.unit_out[u]) outb[u] += t.bytes; else own[u] += t.bytes;
    }
    for (const SOp& s : all.sched) {
      if (!s.live || s.phase != PH_BWD || s.fop < 0) continue;
      const int u = all.fops[s.fop].unit;
      if (u < 0) continue;
      for (int i : s.in)
        if (i >= 0 && all.insts[i].fwd_value && all.insts[i].logical == all.unit_out[u]) self[u] = 1;
    }
    own_pre.assign(nu + 1, 0); out_pre.assign(nu + 1, 0); out_self.assign(nu, 0); ck.assign(nu, 0);
    for (int u = 0; u < nu; ++u) {
      own_pre[u + 1] = own_pre[u] + own[u];
      out_pre[u + 1] = out_pre[u] + outb[u];
      out_self[u] = self[u] ? outb[u] : 0;
      ck[u] = all.tensors[all.unit_in[u]].bytes;
    }
  }
  // bytes units [s, e) hold at the end of their forward pass or replay
  uint64_t saved(int s, int e) const { return (own_pre[e] - own_pre[s]) + (out_pre[e - 1] - out_pre[s]) + out_self[e - 1]; }
  uint64_t total() const { return own_pre.back() + out_pre.back(); }
};

uint64_t model_peak_saved(const Plan& all_stored, const std::vector<int>& seg_begin) {
  const SegModel m(all_stored);
  uint64_t ck = 0, peak = 0;
  for (size_t j = 0; j + 1 < seg_begin.size(); ++j) {
    ck += m.ck[seg_begin[j]];
    peak = std::max(peak, ck + m.saved(seg_begin[j], seg_begin[j + 1]));
  }
  return peak;
}

bool choose_segments(Plan& p) {
  const int nu = (int)p.units.size();
  const int k = p.cfg.k_segments;
  if (k < 1 || k > nu) { p.error = "k_segments must be between 1 and the number of units"; return false; }
  p.seg_begin.assign(1, 0);
  if (p.cfg.boundaries) {
    int prev = 0;
    for (int j = 0; j < k - 1; ++j) {
      int b = p.cfg.boundaries[j];
      if (b <= prev || b >= nu) { p.error = "boundaries must be ascending unit indices in (0, n_units)"; return false; }
      p.seg_begin.push_back(b); prev = b;
    }
    p.seg_begin.push_back(nu);
    return true;
  }
  if (p.cfg.plan_mode == 0 || k == 1) {
    int per = nu / k;
    for (int j = 1; j < k; ++j) p.seg_begin.push_back(j * per);
    p.seg_begin.push_back(nu);
    return true;
  }
  if (p.cfg.plan_mode != 1 && p.cfg.plan_mode != 2) { p.error = "plan_mode must be 0, 1 or 2"; return false; }
  // min-peak: per-unit byte model from the all-stored schedule, then the smallest threshold T for which a
  // partition into k segments exists with  sum_{i<=j} checkpoint_i + saved_j <= T  for every j.
  Plan all = p;
  all.cfg.boundaries = nullptr;
  all.seg_begin = {0, nu};
  if (!build_schedule(all)) { p.error = all.error; return false; }
  const SegModel model(all);
  const std::vector<uint64_t>& ck = model.ck;
  const uint64_t INF = ~0ull;
  std::vector<int> best;
  auto feasible = [&](uint64_t T, std::vector<int>* cuts) {
    // g[j][e]: least checkpoint total with j segments covering units [0, e)
    std::vector<std::vector<uint64_t>> g(k + 1, std::vector<uint64_t>(nu + 1, INF));
    std::vector<std::vector<int>> from(k + 1, std::vector<int>(nu + 1, -1));
    g[0][0] = 0;
    for (int j = 1; j <= k; ++j)
      for (int e = j; e <= nu; ++e)
        for (int s = j - 1; s < e; ++s) {
          if (g[j - 1][s] == INF) continue;
          uint64_t c = g[j - 1][s] + ck[s];
          if (c + model.saved(s, e) > T) continue;
          if (c < g[j][e]) { g[j][e] = c; from[j][e] = s; }
        }
    if (g[k][nu] == INF) return false;
    if (cuts) {
      cuts->assign(k + 1, 0);
      int e = nu;
      for (int j = k; j >= 1; --j) { (*cuts)[j] = e; e = from[j][e]; }
      (*cuts)[0] = 0;
    }
    return true;
  };
  uint64_t lo = 0, hi = model.total();
  for (int u = 0; u < nu; ++u) hi += ck[u];
  while (lo < hi) {
    uint64_t mid = lo + (hi - lo) / 2;
    if (feasible(mid, nullptr)) hi = mid; else lo = mid + 1;
  }
  if (!feasible(lo, &best)) { p.error = "internal: min-peak planner found no partition"; return false; }
  p.seg_begin = best;
  if (p.cfg.plan_mode == 1) return true;

  // plan_mode 2: least recomputation.  The last segment is never replayed, so among the partitions whose modelled
  // peak stays within a threshold the one with the cheapest replay (the forward pass of all segments but the last,
  // from a rough per-unit time estimate) is taken.  The threshold is the minimum peak found above; with a budget it
  // starts at the budget instead and is lowered until the schedule built for the partition fits the budget.
  std::vector<double> cost(nu, 0.0), cpre(nu + 1, 0.0);
  {
    const double rate = p.cfg.precision == OPTORCH_FP32 ? 9e13 : 4.5e14, bw = 4e12, launch = 4e-6, e = (double)p.esize;
    for (const FOp& f : p.fops) {
      if (f.unit < 0) continue;
      const double in_px = (double)f.N * f.H * f.W, out_px = (double)f.N * f.P * f.Q;
      double t = launch;
      if (f.kind == F_CONV) {
        const double w = (double)f.K * f.R * f.S * f.C;
        t += 2.0 * out_px * w / rate + e * (in_px * f.C + out_px * f.K + w) / bw;
      } else if (f.kind == F_BN_APPLY) {
        t += e * out_px * f.C * (f.skip >= 0 ? 3 : 2) / bw;
      } else if (f.kind == F_POOL) {
        t += e * in_px * f.C * 1.25 / bw;
      }
      cost[f.unit] += t;
    }
    for (int u = 0; u < nu; ++u) cpre[u + 1] = cpre[u] + cost[u];
  }
  struct St { uint64_t ck; double cost; int from_s, from_i; };
  auto cheapest = [&](uint64_t T, std::vector<int>* cuts) {
    // per (segments used, units covered): the states no other state beats in both checkpoint bytes and replay cost
    std::vector<std::vector<std::vector<St>>> S(k + 1, std::vector<std::vector<St>>(nu + 1));
    S[0][0].push_back(St{0, 0.0, -1, -1});
    for (int j = 1; j <= k; ++j)
      for (int e = j; e <= nu - (k - j); ++e) {
        if (j == k && e != nu) continue;
        std::vector<St> cand;
        for (int s0 = j - 1; s0 < e; ++s0)
          for (size_t i = 0; i < S[j - 1][s0].size(); ++i) {
            const St& st = S[j - 1][s0][i];
            const uint64_t c = st.ck + ck[s0];
            if (c + model.saved(s0, e) > T) continue;
            cand.push_back(St{c, st.cost + (e == nu ? 0.0 : cpre[e] - cpre[s0]), s0, (int)i});
          }
        std::sort(cand.begin(), cand.end(), [](const St& a, const St& b) { return a.ck != b.ck ? a.ck < b.ck : a.cost < b.cost; });
        double least = 1e300;
        for (const St& c : cand)
          if (c.cost < least) { S[j][e].push_back(c); least = c.cost; }
      }
    if (S[k][nu].empty()) return false;
    size_t bi = 0;
    for (size_t i = 1; i < S[k][nu].size(); ++i)
      if (S[k][nu][i].cost < S[k][nu][bi].cost) bi = i;
    cuts->assign(k + 1, 0);
    int e = nu; size_t idx = bi;
    for (int j = k; j >= 1; --j) {
      (*cuts)[j] = e;
      const St& st = S[j][e][idx];
      e = st.from_s; idx = (size_t)st.from_i;
    }
    return true;
  };
  const uint64_t budget = p.cfg.activation_budget_bytes;
  if (!budget) {
    std::vector<int> cuts;
    if (cheapest(lo, &cuts)) { p.seg_begin = cuts; return true; }
    p.seg_begin = best;
    return true;
  }
  // With a budget: the modelled peak (saved tensors only) of a partition is below its arena (transients, alignment,
  // fragmentation), so the threshold that just fits the budget is searched: lowered in sixteenths from the budget until
  // the scheduled arena fits, then bisected between that threshold and the last one that did not.
  auto fits = [&](uint64_t T, std::vector<int>* cuts, bool* error) {
    *error = false;
    if (!cheapest(T, cuts)) return false;
    Plan trial = p;
    trial.cfg.boundaries = nullptr;
    trial.seg_begin = *cuts;
    if (!build_schedule(trial)) { p.error = trial.error; *error = true; return false; }
    return trial.arena_bytes <= budget;
  };
  uint64_t T = budget > lo ? budget : lo, too_big = 0;
  std::vector<int> good;
  uint64_t good_T = 0;
  for (int attempt = 0; attempt < 24; ++attempt) {
    std::vector<int> cuts;
    bool error;
    if (fits(T, &cuts, &error)) { good = cuts; good_T = T; break; }
    if (error) return false;
    too_big = T;
    if (T == lo) break;
    T = std::max<uint64_t>(lo, T - T / 16);
  }
  if (!good.empty()) {
    for (int it = 0; it < 8 && too_big > good_T + (budget >> 10); ++it) {
      const uint64_t mid = good_T + (too_big - good_T) / 2;
      std::vector<int> cuts;
      bool error;
      if (fits(mid, &cuts, &error)) { good = cuts; good_T = mid; }
      else { if (error) return false; too_big = mid; }
    }
    p.seg_begin = good;
    return true;
  }
  p.seg_begin = best;  // nothing cheaper fits: the minimum-peak partition
  return true;
}

}  // namespace oseq
