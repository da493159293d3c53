"""CPU oracle for one training step of a sequential CNN.  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the CPU-baseline leg of the benchmark may use
this module; the product path never does.  It shares no code with the HIP
library.

What it computes.  The paper's sequential-checkpoint scheme (Section
"Sequential-checkpoint training", and the Introduction's description of
segments) stores only segment inputs and re-runs each segment's forward pass
during back-propagation; the recomputed activations equal the ones a standard
pipeline would have stored, so the gradients are exactly those of ordinary
back-propagation.  The oracle is therefore that plain definition written out:
a forward pass that keeps every activation, followed by reverse-mode
differentiation, in float64 (float32 on request, for timing), plus one
SGD-momentum update.  The plain path has no checkpointing, no loss scaling and
no half precision: mixed precision (Section "Mixed-precision training") changes
the storage type, not the function being differentiated.

Layer definitions are the textbook ones (the paper delegates layer math to its
host framework; the neuron/back-propagation primer in the same section is the
only description):

  conv      cross-correlation, zero padding, stride, NHWC activations and
            (C_out, kh, kw, C_in) weights, optional bias
  BN        training mode, per channel over batch*H*W, biased variance,
            y = gamma * (z - mean) * rstd + beta
  ReLU      max(y, 0); derivative 0 at y == 0
  residual  out = relu(F(x) + shortcut(x)); projection shortcut = 1x1 conv + BN
  maxpool   2x2 stride 2; gradient goes to the first maximum in scan order
  GAP       mean over H*W
  loss      mean over the batch of logsumexp(logits) - logits[label]
  SGD       v <- mu*v + g ; w <- w - lr*v

matmul / tensordot from numpy serve as the contraction step of a convolution
tap; nothing is blocked, fused or reordered.

Storage emulation (optional).  A ReLU mask is an integer decision taken by a
floating-point comparison, and a 16-bit pipeline takes it on 16-bit values.  So
that both sides take it in the same precision, `loss_and_grads(storage="bf16" |
"fp16", loss_scale=S)` follows the mixed-precision recipe (Section
"Mixed-precision training": 16-bit storage, 32-bit arithmetic) as "every tensor
kept in 16 bits is rounded to nearest even exactly once, when it is stored":
the input image, the 16-bit copy of each convolution weight, each convolution
output in front of a BatchNorm (the statistics are then those of the stored
values), each unit's and each layer's output activation, and each activation
gradient (the gradient entering the network body, the gradient behind each
BatchNorm, and the gradient w.r.t. each layer's input; where two paths meet, the
sum is the stored tensor).  The loss gradient is multiplied by S and the
parameter gradients divided by S at the end.  Everything between two stored
tensors (contractions, BatchNorm statistics and sums, the loss head, parameter
gradients) stays in float64.  With storage=None the hooks are the identity and
the function is the plain definition.  The placement of the rounding points is
pinned by worked examples (tests/golden/mixed_precision_worked.txt).

Inference mode.  BatchNorm keeps running estimates of each channel's mean and variance (exponential averages of the
batch mean and of the unbiased batch variance, momentum 0.1, started at 0 and 1) and `predict` evaluates the network
with those in place of the batch statistics: y = gamma * (z - running_mean) / sqrt(running_var + eps) + beta.  The
paper trains and then evaluates its networks (Section "Results", accuracy after ten epochs)
with a framework's BatchNorm; these are that layer's standard definitions.

Pins (tests/test_oracle_pins.py): central finite differences on every layer
kind, closed forms of the loss and the update, BatchNorm orthogonality
invariants, reduction of 1x1 conv to a matrix product, agreement with
scipy.signal.correlate2d, brute-force Jacobians of the convolution, batch
permutation symmetry.
"""
from __future__ import annotations

import numpy as np

CONV, MAXPOOL2, BASIC_BLOCK, BOTTLENECK, GAP_LINEAR_CE, FLATTEN_LINEAR_CE = range(6)
BN_EPS = 1e-5


# ------------------------------------------------------ 16-bit storage ------
def round_to_bf16(a):
    """Round to the nearest bfloat16 (ties to even), returned in the input dtype."""
    a32 = np.ascontiguousarray(a, dtype=np.float32)
    u = a32.view(np.uint32)
    r = ((u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) & np.uint32(0xFFFF0000)).view(np.float32)
    r = np.where(np.isnan(a32), np.float32(np.nan), r)
    return r.astype(np.asarray(a).dtype if np.asarray(a).dtype.kind == "f" else np.float64)


def round_to_fp16(a):
    """Round to the nearest IEEE half (ties to even; overflow gives inf), returned in the input dtype."""
    with np.errstate(over="ignore"):
        r = np.asarray(a, dtype=np.float32).astype(np.float16)
    return r.astype(np.asarray(a).dtype if np.asarray(a).dtype.kind == "f" else np.float64)


def _quantizer(storage):
    if storage is None:
        return lambda a: a
    if storage == "bf16":
        return round_to_bf16
    if storage == "fp16":
        return round_to_fp16
    raise ValueError("storage must be None, 'bf16' or 'fp16'")


# ---------------------------------------------------------------- layers ----
def conv2d_forward(x, w, b, stride, pad):
    """z[n,p,q,k] = b[k] + sum_{r,s,c} x[n, p*stride+r-pad, q*stride+s-pad, c] * w[k,r,s,c]."""
    n, h, wd, c = x.shape
    k, r_, s_, _ = w.shape
    p = (h + 2 * pad - r_) // stride + 1
    q = (wd + 2 * pad - s_) // stride + 1
    xp = np.zeros((n, h + 2 * pad, wd + 2 * pad, c), dtype=x.dtype)
    xp[:, pad:pad + h, pad:pad + wd, :] = x
    z = np.zeros((n, p, q, k), dtype=x.dtype)
    for r in range(r_):
        for s in range(s_):
            xs = xp[:, r:r + stride * (p - 1) + 1:stride, s:s + stride * (q - 1) + 1:stride, :]
            z += np.matmul(xs, w[:, r, s, :].T)
    if b is not None:
        z += b
    return z


def conv2d_backward(x, w, dz, stride, pad, has_bias):
    """Returns (dx, dw, db) for z = conv2d_forward(x, w, b)."""
    n, h, wd, c = x.shape
    k, r_, s_, _ = w.shape
    _, p, q, _ = dz.shape
    xp = np.zeros((n, h + 2 * pad, wd + 2 * pad, c), dtype=x.dtype)
    xp[:, pad:pad + h, pad:pad + wd, :] = x
    dxp = np.zeros_like(xp)
    dw = np.zeros_like(w)
    for r in range(r_):
        for s in range(s_):
            sl = (slice(None), slice(r, r + stride * (p - 1) + 1, stride),
                  slice(s, s + stride * (q - 1) + 1, stride), slice(None))
            dw[:, r, s, :] = np.tensordot(dz, xp[sl], axes=([0, 1, 2], [0, 1, 2]))
            dxp[sl] += np.matmul(dz, w[:, r, s, :])
    dx = dxp[:, pad:pad + h, pad:pad + wd, :]
    db = dz.sum(axis=(0, 1, 2)) if has_bias else None
    return dx, dw, db


def batchnorm_forward(z, gamma, beta, eps=BN_EPS):
    mean = z.mean(axis=(0, 1, 2))
    var = ((z - mean) ** 2).mean(axis=(0, 1, 2))
    rstd = 1.0 / np.sqrt(var + eps)
    xhat = (z - mean) * rstd
    return gamma * xhat + beta, (xhat, rstd)


def batchnorm_eval(z, gamma, beta, running_mean, running_var, eps=BN_EPS):
    """Inference-mode BatchNorm: the running estimates take the place of the batch statistics."""
    return gamma * (z - running_mean) / np.sqrt(running_var + eps) + beta


def batchnorm_running_update(running_mean, running_var, batch_mean, batch_var_biased, count, momentum=0.1):
    """Exponential averages of the batch mean and of the unbiased batch variance (count = batch * H * W)."""
    unbiased = batch_var_biased * count / (count - 1) if count > 1 else batch_var_biased
    return ((1.0 - momentum) * running_mean + momentum * batch_mean,
            (1.0 - momentum) * running_var + momentum * unbiased)


def batchnorm_backward(dy, cache, gamma):
    xhat, rstd = cache
    m = dy.shape[0] * dy.shape[1] * dy.shape[2]
    dbeta = dy.sum(axis=(0, 1, 2))
    dgamma = (dy * xhat).sum(axis=(0, 1, 2))
    dz = (gamma * rstd / m) * (m * dy - dbeta - xhat * dgamma)
    return dz, dgamma, dbeta


def relu_forward(y):
    return np.maximum(y, 0)


def relu_backward(da, y):
    return da * (y > 0)


def maxpool2_forward(x):
    n, h, w, c = x.shape
    win = np.stack([x[:, 0:h - h % 2:2, 0:w - w % 2:2, :], x[:, 0:h - h % 2:2, 1:w:2, :],
                    x[:, 1:h:2, 0:w - w % 2:2, :], x[:, 1:h:2, 1:w:2, :]], axis=0)
    arg = win.argmax(axis=0)  # first maximum in (row, col) scan order
    return win.max(axis=0), arg


def maxpool2_backward(dy, arg, xshape):
    dx = np.zeros(xshape, dtype=dy.dtype)
    n, h, w, c = xshape
    for i, (dr, dc) in enumerate(((0, 0), (0, 1), (1, 0), (1, 1))):
        dx[:, dr:h - h % 2:2, dc:w - w % 2:2, :] += dy * (arg == i)
    return dx


def softmax_ce_forward(logits, y):
    """Mean over the batch of logsumexp(logits_n) - logits_n[y_n] (max-shifted)."""
    mx = logits.max(axis=1, keepdims=True)
    lse = mx[:, 0] + np.log(np.exp(logits - mx).sum(axis=1))
    b = logits.shape[0]
    loss = (lse - logits[np.arange(b), y]).sum() / b
    prob = np.exp(logits - lse[:, None])
    return loss, prob


def softmax_ce_backward(prob, y):
    b = prob.shape[0]
    d = prob.copy()
    d[np.arange(b), y] -= 1.0
    return d / b


def sgd_momentum_step(w, v, g, lr, momentum):
    """v <- momentum*v + g ; w <- w - lr*v.  Returns (w_new, v_new)."""
    v_new = momentum * v + g
    return w - lr * v_new, v_new


def loss_scale_update(scale, clean_steps, found_inf, growth_interval, growth=2.0, backoff=0.5):
    """Dynamic loss-scale state machine of mixed-precision training (the paper cites the
    standard recipe in Section "Mixed-precision training"): on a non-finite gradient the
    step is skipped and the scale is multiplied by `backoff`; after `growth_interval`
    consecutive finite steps it is multiplied by `growth`.
    Returns (scale, clean_steps, step_skipped)."""
    if found_inf:
        return scale * backoff, 0, True
    clean_steps += 1
    if clean_steps == growth_interval:
        return scale * growth, 0, False
    return scale, clean_steps, False


# ------------------------------------------------------------- network ------
class _Params:
    """Sequential reader over the flat parameter vector; the writer side collects gradients."""

    def __init__(self, flat, q=lambda a: a, flips=None, kink_tau=None):
        self.flat, self.off, self.q = flat, 0, q
        self.relu_count = 0           # ReLU layers are numbered in forward order
        self.flips = flips or {}      # {relu number: (flat indices, decisions forced there)}
        self.kink_tau, self.kinks = kink_tau, []
        self.moments = {}             # {flat offset of a BatchNorm's gamma: (batch mean, biased variance, count)}
        self.running = None           # inference mode: {flat offset of gamma: (running mean, running variance)}

    def take(self, shape):
        n = int(np.prod(shape))
        v = self.flat[self.off:self.off + n].reshape(shape)
        self.off += n
        return v


def _cbr_forward(x, pr, cin, cout, k, stride, pad, bn, relu, bias, skip=None):
    """conv [+bias] [+BN] [+skip] [+ReLU]; returns (out, cache)."""
    q = pr.q
    w = q(pr.take((cout, k, k, cin)))  # 16-bit copy of the master weights
    b = pr.take((cout,)) if bias else None
    z = conv2d_forward(x, w, b, stride, pad)
    cache = {"x": x, "w": w, "stride": stride, "pad": pad, "bias": bias, "bn": bn, "relu": relu, "q": q}
    y = z
    shift_off = pr.off - cout if bias else -1  # flat index of the per-channel additive parameter in front of the ReLU
    if bn:
        gamma, beta = pr.take((cout,)), pr.take((cout,))
        shift_off = pr.off - cout
        z = q(z)  # the convolution output is a stored tensor; statistics are taken from what is stored
        if pr.running is not None:
            y = batchnorm_eval(z, gamma, beta, *pr.running[shift_off - cout])
        else:
            y, cache["bn_cache"] = batchnorm_forward(z, gamma, beta)
            mean = z.mean(axis=(0, 1, 2))
            pr.moments[shift_off - cout] = (mean, ((z - mean) ** 2).mean(axis=(0, 1, 2)),
                                            z.shape[0] * z.shape[1] * z.shape[2])
        cache["gamma"] = gamma
    if skip is not None:
        y = y + skip
    cache["y"] = y
    if relu:
        rid = pr.relu_count
        pr.relu_count += 1
        mask = y > 0
        if pr.kink_tau is not None:  # decisions within kink_tau x rms(y) of the kink
            near = np.flatnonzero(np.abs(y).ravel() < pr.kink_tau * np.sqrt(np.mean(y * y)))
            pr.kinks += [(rid, int(i), (shift_off + int(i) % cout) if shift_off >= 0 else -1, bool(mask.ravel()[i]))
                         for i in near]
        if rid in pr.flips:
            mask = mask.copy()
            mask.ravel()[np.asarray(pr.flips[rid][0], dtype=np.int64)] = np.asarray(pr.flips[rid][1], dtype=bool)
        cache["mask"] = mask
    return q(relu_forward(y) if relu else y), cache


def _cbr_backward(da, cache, grads):
    """Returns (dx, dskip); appends this layer's parameter gradients to `grads` (in layout order).
    dx is the raw data gradient: the caller adds any second contribution and then stores (rounds) it."""
    dy = da * cache["mask"] if cache["relu"] else da  # relu_backward with the recorded decisions
    dskip = dy
    g_bn = []
    if cache["bn"]:
        dz, dgamma, dbeta = batchnorm_backward(dy, cache["bn_cache"], cache["gamma"])
        dz = cache["q"](dz)
        g_bn = [dgamma, dbeta]
    else:
        dz = dy
    dx, dw, db = conv2d_backward(cache["x"], cache["w"], dz, cache["stride"], cache["pad"], cache["bias"])
    grads.append([dw] + ([db] if cache["bias"] else []) + g_bn)
    return dx, dskip


def _unit_forward(u, x, pr):
    if u.kind == CONV:
        out, c = _cbr_forward(x, pr, u.cin, u.cout, u.ksize, u.stride, u.pad, u.has_bn, u.has_relu, u.has_bias)
        return out, ("conv", c)
    if u.kind == MAXPOOL2:
        out, arg = maxpool2_forward(x)
        return out, ("pool", arg, x.shape)
    if u.kind in (BASIC_BLOCK, BOTTLENECK):
        proj = (u.cin != u.cout) or (u.stride != 1)
        if u.kind == BASIC_BLOCK:
            a1, c1 = _cbr_forward(x, pr, u.cin, u.cout, 3, u.stride, 1, 1, 1, 0)
            main_in, caches, last = a1, [c1], (u.cout, u.cout, 3, 1, 1)
        else:
            mid = u.cout // 4
            a1, c1 = _cbr_forward(x, pr, u.cin, mid, 1, 1, 0, 1, 1, 0)
            a2, c2 = _cbr_forward(a1, pr, mid, mid, 3, u.stride, 1, 1, 1, 0)
            main_in, caches, last = a2, [c1, c2], (mid, u.cout, 1, 1, 0)
        # the last conv's parameters come before the shortcut's in the flat layout, but its
        # forward needs the shortcut's output: read the parameter views in layout order first
        lw_off = pr.off
        n_last = last[1] * last[2] * last[2] * last[0] + 2 * last[1]
        pr.off += n_last
        if proj:
            sc, csc = _cbr_forward(x, pr, u.cin, u.cout, 1, u.stride, 0, 1, 0, 0)
        else:
            sc, csc = x, None
        end_off = pr.off
        pr.off = lw_off
        out, cl = _cbr_forward(main_in, pr, last[0], last[1], last[2], last[3], last[4], 1, 1, 0, skip=sc)
        pr.off = end_off
        return out, ("block", caches + [cl], csc)
    raise ValueError("unit kind %r is not a body unit" % (u.kind,))


def _unit_backward(cache, da, grads):
    tag = cache[0]
    if tag == "conv":
        dx, _ = _cbr_backward(da, cache[1], grads)
        return cache[1]["q"](dx)
    if tag == "pool":
        return maxpool2_backward(da, cache[1], cache[2])
    caches, csc = cache[1], cache[2]
    q = caches[0]["q"]
    local = []
    d, dskip = _cbr_backward(da, caches[-1], local)
    for c in reversed(caches[:-1]):
        d, _ = _cbr_backward(q(d), c, local)
    local.reverse()  # conv1, conv2, [conv3]
    if csc is not None:
        dsc, _ = _cbr_backward(dskip, csc, local)  # appended last = layout order
        d = q(d + dsc)  # the gradient w.r.t. the block's input is one stored tensor: the sum, rounded once
    else:
        d = q(d + dskip)
    grads.append([g for layer in local for g in layer])
    return d


def loss_and_grads(units, params, x, y, dtype=np.float64, return_trace=False, storage=None, loss_scale=1.0,
                   flips=None, kink_tau=None):
    """Loss and flat parameter gradient of the network `units` at `params` on the batch (x, y).

    units  : sequence of objects with attributes kind, cin, cout, ksize, stride, pad,
             has_bn, has_relu, has_bias; the last one is the loss head
    params : flat vector in layout order (unit order; conv weight, [bias], gamma, beta;
             linear weight (classes x features), bias)
    x      : (B, H, W, C) images;  y : (B,) integer labels
    storage, loss_scale : 16-bit storage emulation, see the module docstring; the returned
             gradients are unscaled (non-finite if a stored value overflowed)
    return_trace : a third return value holds the stored tensors: {"input": the batch as stored, "units": the
             output of every body unit, "logits", "d_units": the gradient w.r.t. the input of every unit (entry i
             for unit i; the last entry is the gradient entering the body from the head), scaled by loss_scale}
    kink_tau : if given, a third return value lists the ReLU decisions whose pre-activation lies within
             kink_tau x rms of zero -- decisions a finite-precision evaluation may legitimately take the
             other way -- as (relu number, flat index into that layer's output, flat index of the gradient
             entry of the BatchNorm shift / bias of that channel, which such a decision changes directly,
             the decision taken here)
    flips  : {relu number: (indices, decisions)} -- back-propagate with those decisions forced to the
             given values (forward unchanged)
    """
    q = _quantizer(storage)
    params = np.asarray(params, dtype=dtype)
    a = q(np.asarray(x, dtype=dtype))
    y = np.asarray(y).astype(np.int64)
    pr = _Params(params, q, flips, kink_tau)
    caches = []
    trace = {"input": a, "units": [], "d_units": []}
    for u in units[:-1]:
        a, c = _unit_forward(u, a, pr)
        caches.append(c)
        if return_trace:
            trace["units"].append(a)
    head = units[-1]
    if head.kind == GAP_LINEAR_CE:
        feat = a.mean(axis=(1, 2))
    elif head.kind == FLATTEN_LINEAR_CE:
        feat = a.reshape(a.shape[0], -1)
    else:
        raise ValueError("the last unit must be a loss head")
    wl = pr.take((head.cout, feat.shape[1]))
    bl = pr.take((head.cout,))
    if pr.off != params.size:
        raise ValueError("parameter vector has %d entries, network needs %d" % (params.size, pr.off))
    logits = feat @ wl.T + bl
    loss, prob = softmax_ce_forward(logits, y)
    trace["logits"] = logits

    dlogits = softmax_ce_backward(prob, y) * loss_scale
    dwl = dlogits.T @ feat
    dbl = dlogits.sum(axis=0)
    dfeat = dlogits @ wl
    if head.kind == GAP_LINEAR_CE:
        hw = a.shape[1] * a.shape[2]
        da = np.broadcast_to(dfeat[:, None, None, :] / hw, a.shape).astype(dtype)
    else:
        da = dfeat.reshape(a.shape)
    da = q(da)
    trace["d_units"].append(da)
    grads_rev = [[dwl, dbl]]
    for c in reversed(caches):
        before = len(grads_rev)
        da = _unit_backward(c, da, grads_rev)
        trace["d_units"].append(da)
        if len(grads_rev) == before:
            grads_rev.append([])
    flat = [np.ravel(g) for unit_g in reversed(grads_rev) for g in unit_g]
    grad = np.concatenate(flat) if flat else np.zeros(0, dtype)
    assert grad.size == params.size
    if loss_scale != 1.0:
        grad = grad / loss_scale
    if return_trace:
        trace["d_units"].reverse()  # d_units[i]: gradient w.r.t. the input of unit i, as stored (scaled by loss_scale)
        return float(loss), grad, trace
    if kink_tau is not None:
        return float(loss), grad, pr.kinks
    return float(loss), grad


def train_step(units, params, velocity, x, y, lr, momentum, dtype=np.float64):
    """One SGD-momentum step; returns (loss, grads, new_params, new_velocity)."""
    loss, g = loss_and_grads(units, params, x, y, dtype)
    w, v = sgd_momentum_step(np.asarray(params, dtype), np.asarray(velocity, dtype), g, lr, momentum)
    return loss, g, w, v



# ------------------------------------------------- running statistics, inference ------
def _forward_logits(units, pr, a):
    for u in units[:-1]:
        a, _ = _unit_forward(u, a, pr)
    head = units[-1]
    if head.kind == GAP_LINEAR_CE:
        feat = a.mean(axis=(1, 2))
    elif head.kind == FLATTEN_LINEAR_CE:
        feat = a.reshape(a.shape[0], -1)
    else:
        raise ValueError("the last unit must be a loss head")
    wl = pr.take((head.cout, feat.shape[1]))
    bl = pr.take((head.cout,))
    return feat @ wl.T + bl


def forward_trace(units, params, x, dtype=np.float64, storage=None):
    """The training-mode forward pass alone (batch statistics in every BatchNorm): {"input": the batch as stored,
    "units": the output of every body unit, "logits"}; storage as in loss_and_grads."""
    q = _quantizer(storage)
    pr = _Params(np.asarray(params, dtype=dtype), q)
    a = q(np.asarray(x, dtype=dtype))
    trace = {"input": a, "units": []}
    for u in units[:-1]:
        a, _ = _unit_forward(u, a, pr)
        trace["units"].append(a)
    head = units[-1]
    feat = a.mean(axis=(1, 2)) if head.kind == GAP_LINEAR_CE else a.reshape(a.shape[0], -1)
    wl = pr.take((head.cout, feat.shape[1]))
    bl = pr.take((head.cout,))
    trace["logits"] = feat @ wl.T + bl
    return trace


def initial_running_stats(units, params, x_shape):
    """Flat vector of running statistics before the first step: per BatchNorm, in parameter-layout order, C zeros
    (mean) then C ones (variance)."""
    moments = batch_moments(units, params, np.zeros(x_shape))
    return np.concatenate([np.concatenate([np.zeros_like(m[0]), np.ones_like(m[1])]) for m in moments]) \
        if moments else np.zeros(0)


def batch_moments(units, params, x, dtype=np.float64, storage=None):
    """Per BatchNorm, in parameter-layout order: (batch mean, biased batch variance, count) of its input on x."""
    q = _quantizer(storage)
    pr = _Params(np.asarray(params, dtype=dtype), q)
    _forward_logits(units, pr, q(np.asarray(x, dtype=dtype)))
    return [pr.moments[k] for k in sorted(pr.moments)]


def update_running_stats(running, moments, momentum=0.1):
    """One training step's update of the flat running-statistics vector from that step's batch moments."""
    out, off = [], 0
    for mean, var, count in moments:
        c = mean.size
        rm, rv = batchnorm_running_update(running[off:off + c], running[off + c:off + 2 * c], mean, var, count, momentum)
        out += [rm, rv]
        off += 2 * c
    return np.concatenate(out) if out else np.zeros(0)


def predict(units, params, running, x, dtype=np.float64, storage=None):
    """Logits of the network in inference mode: BatchNorm uses the running statistics `running` (flat, layout as in
    initial_running_stats); storage as in loss_and_grads."""
    q = _quantizer(storage)
    params = np.asarray(params, dtype=dtype)
    # the keys (flat offsets of the gammas, ascending) are those a batch-mode pass records
    keys = sorted(_moment_keys(units, params, np.asarray(x).shape))
    pr = _Params(params, q)
    pr.running, off = {}, 0
    for k, c in keys:
        pr.running[k] = (np.asarray(running[off:off + c], dtype), np.asarray(running[off + c:off + 2 * c], dtype))
        off += 2 * c
    return _forward_logits(units, pr, q(np.asarray(x, dtype=dtype)))


def _moment_keys(units, params, x_shape):
    pr = _Params(params)
    _forward_logits(units, pr, np.zeros((1,) + tuple(x_shape[1:]), dtype=params.dtype))
    return [(k, v[0].size) for k, v in pr.moments.items()]

