"""Seeded synthetic workloads: network descriptions and input generators.

This module holds no arithmetic of the training step itself.  It only
describes networks as lists of units (the atomic pieces a checkpoint
boundary may fall between) and draws pixels, labels and initial weights
from a seeded generator.  Both the HIP path and the CPU oracle are fed
from here; neither imports the other.

Unit kinds (integer codes are the ones the C ABI uses):

    CONV               conv kxk [+bias] [+BatchNorm] [+ReLU]
    MAXPOOL2           2x2 max-pool, stride 2
    BASIC_BLOCK        conv3x3-BN-ReLU, conv3x3-BN, (+shortcut), ReLU
    BOTTLENECK         conv1x1-BN-ReLU, conv3x3-BN-ReLU, conv1x1-BN, (+shortcut), ReLU
    GAP_LINEAR_CE      global average pool, linear, softmax cross-entropy
    FLATTEN_LINEAR_CE  NHWC flatten, linear, softmax cross-entropy

The synthetic images copy the shape of the paper's CIFAR experiments
(Section "Results": 32x32x3 colour images, 10 classes; 100 classes for the
CIFAR-100 claim in the abstract); the datasets themselves are not used.
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import Dict, List, Sequence, Tuple

import numpy as np

CONV = 0
MAXPOOL2 = 1
BASIC_BLOCK = 2
BOTTLENECK = 3
GAP_LINEAR_CE = 4
FLATTEN_LINEAR_CE = 5

FP32 = 0
BF16 = 1
FP16 = 2

MASTER_SEED = 210500619


@dataclass(frozen=True)
class Unit:
    kind: int
    cin: int = 0
    cout: int = 0
    ksize: int = 0
    stride: int = 1
    pad: int = 0
    has_bn: int = 0
    has_relu: int = 0
    has_bias: int = 0


def conv(cin, cout, ksize=3, stride=1, pad=None, bn=True, relu=True, bias=None) -> Unit:
    if pad is None:
        pad = ksize // 2
    if bias is None:
        bias = not bn
    return Unit(CONV, cin, cout, ksize, stride, pad, int(bn), int(relu), int(bias))


def maxpool() -> Unit:
    return Unit(MAXPOOL2, ksize=2, stride=2)


def basic_block(cin, cout, stride=1) -> Unit:
    return Unit(BASIC_BLOCK, cin, cout, 3, stride, 1, 1, 1, 0)


def bottleneck(cin, cout, stride=1) -> Unit:
    return Unit(BOTTLENECK, cin, cout, 3, stride, 1, 1, 1, 0)


def gap_linear_ce(features, classes) -> Unit:
    return Unit(GAP_LINEAR_CE, features, classes, has_bias=1)


def flatten_linear_ce(channels, classes) -> Unit:
    """`channels` is C of the incoming H x W x C map; the linear layer sees H*W*C features."""
    return Unit(FLATTEN_LINEAR_CE, channels, classes, has_bias=1)


# --------------------------------------------------------------------------
# network builders
# --------------------------------------------------------------------------
def tiny_cnn(classes=10) -> List[Unit]:
    return [conv(3, 8, bn=False), conv(8, 8, bn=False), gap_linear_ce(8, classes)]


def vgg11_bn(classes=10) -> List[Unit]:
    widths = [64, "M", 128, "M", 256, 256, "M", 512, 512, "M", 512, 512, "M"]
    units, c = [], 3
    for w in widths:
        if w == "M":
            units.append(maxpool())
        else:
            units.append(conv(c, w))
            c = w
    units.append(flatten_linear_ce(c, classes))
    return units


def resnet_basic(stages: Sequence[int], classes=100, base=64) -> List[Unit]:
    units, c = [conv(3, base)], base
    for si, nb in enumerate(stages):
        cout = base << si
        for bi in range(nb):
            units.append(basic_block(c, cout, 2 if (bi == 0 and si > 0) else 1))
            c = cout
    units.append(gap_linear_ce(c, classes))
    return units


def resnet_bottleneck(stages: Sequence[int], classes=100, base=64) -> List[Unit]:
    units, c = [conv(3, base)], base
    for si, nb in enumerate(stages):
        cout = (base * 4) << si
        for bi in range(nb):
            units.append(bottleneck(c, cout, 2 if (bi == 0 and si > 0) else 1))
            c = cout
    units.append(gap_linear_ce(c, classes))
    return units


@dataclass(frozen=True)
class Workload:
    name: str
    units: Tuple[Unit, ...]
    batch: int
    height: int
    width: int
    channels: int
    classes: int
    precision: int
    k_segments: int
    momentum: float
    loss_scale_init: float
    pixels: str  # "uniform" or "gauss"
    budget_bytes: int = 0
    plan_mode: int = 0  # how segment boundaries are chosen: 0 equal unit count, 1 least peak of saved bytes, 2 least
    #                     recomputation within that peak (or within budget_bytes); the benchmark networks use 2
    seed: int = MASTER_SEED


def config(index: int, batch: int | None = None, size: int | None = None) -> Workload:
    """The five benchmark configurations (index 1..5) and, as index 6, the shape of the paper's memory experiment
    (Section "Results": 16 images of 512 x 512 x 3 through ResNet-18): large images, tiny
    batch.  `batch` overrides the batch size, `size` the image height and width."""
    if index == 1:
        w = Workload("tiny_cnn_fp32_k2", tuple(tiny_cnn(10)), 8, 32, 32, 3, 10, FP32, 2, 0.0, 1.0, "uniform")
    elif index == 2:
        w = Workload("vgg11_bn_fp32_k4", tuple(vgg11_bn(10)), 128, 32, 32, 3, 10, FP32, 4, 0.0, 1.0, "gauss", plan_mode=2)
    elif index == 3:
        w = Workload("resnet18_bf16_k4", tuple(resnet_basic([2, 2, 2, 2], 100)), 256, 32, 32, 3, 100,
                     BF16, 4, 0.9, 1.0, "gauss", plan_mode=2)
    elif index == 4:
        w = Workload("resnet50_fp16_k8", tuple(resnet_bottleneck([3, 4, 6, 3], 100)), 512, 32, 32, 3, 100,
                     FP16, 8, 0.0, 65536.0, "gauss", plan_mode=2)
    elif index == 5:
        w = Workload("resnet152_bf16_k7", tuple(resnet_bottleneck([3, 8, 36, 3], 100)), 4096, 32, 32, 3, 100,
                     BF16, 7, 0.0, 1.0, "gauss", budget_bytes=32 << 30, plan_mode=2)
    elif index == 6:
        w = Workload("resnet18_fp32_k4_512px", tuple(resnet_basic([2, 2, 2, 2], 10)), 16, 512, 512, 3, 10,
                     FP32, 4, 0.0, 1.0, "gauss", plan_mode=2)
    else:
        raise ValueError("config index must be 1..6")
    if batch is not None:
        w = Workload(**{**w.__dict__, "batch": int(batch)})
    if size is not None:
        w = Workload(**{**w.__dict__, "height": int(size), "width": int(size)})
    return Workload(**{**w.__dict__, "seed": MASTER_SEED + index})


# --------------------------------------------------------------------------
# parameter layout (flat fp32 arena order) -- shapes only, no arithmetic
# --------------------------------------------------------------------------
def _conv_entries(prefix, cin, cout, k, bn, bias):
    out = [(prefix + ".w", (cout, k, k, cin), "conv_w", k * k * cin)]
    if bias:
        out.append((prefix + ".b", (cout,), "bias", 0))
    if bn:
        out.append((prefix + ".gamma", (cout,), "gamma", 0))
        out.append((prefix + ".beta", (cout,), "beta", 0))
    return out


def param_layout(units: Sequence[Unit], height: int, width: int) -> List[Tuple[str, Tuple[int, ...], str, int]]:
    """(name, shape, role, fan_in) of every parameter tensor, in flat-arena order.

    Order: unit order; inside a unit conv weight (C_out, kh, kw, C_in), [bias],
    BN gamma, BN beta; inside a residual block conv1.., conv2.., [conv3..],
    then the projection shortcut if the block has one; linear weight
    (classes x features) then bias.
    """
    out = []
    h, w = height, width
    for ui, u in enumerate(units):
        p = "u%d" % ui
        if u.kind == CONV:
            out += _conv_entries(p, u.cin, u.cout, u.ksize, u.has_bn, u.has_bias)
            h = (h + 2 * u.pad - u.ksize) // u.stride + 1
            w = (w + 2 * u.pad - u.ksize) // u.stride + 1
        elif u.kind == MAXPOOL2:
            h, w = h // 2, w // 2
        elif u.kind == BASIC_BLOCK:
            out += _conv_entries(p + ".c1", u.cin, u.cout, 3, 1, 0)
            out += _conv_entries(p + ".c2", u.cout, u.cout, 3, 1, 0)
            if u.cin != u.cout or u.stride != 1:
                out += _conv_entries(p + ".sc", u.cin, u.cout, 1, 1, 0)
            h = (h + 2 - 3) // u.stride + 1
            w = (w + 2 - 3) // u.stride + 1
        elif u.kind == BOTTLENECK:
            mid = u.cout // 4
            out += _conv_entries(p + ".c1", u.cin, mid, 1, 1, 0)
            out += _conv_entries(p + ".c2", mid, mid, 3, 1, 0)
            out += _conv_entries(p + ".c3", mid, u.cout, 1, 1, 0)
            if u.cin != u.cout or u.stride != 1:
                out += _conv_entries(p + ".sc", u.cin, u.cout, 1, 1, 0)
            h = (h + 2 - 3) // u.stride + 1
            w = (w + 2 - 3) // u.stride + 1
        elif u.kind in (GAP_LINEAR_CE, FLATTEN_LINEAR_CE):
            feat = u.cin if u.kind == GAP_LINEAR_CE else h * w * u.cin
            out.append((p + ".lin.w", (u.cout, feat), "lin_w", feat))
            out.append((p + ".lin.b", (u.cout,), "bias", 0))
        else:
            raise ValueError("unknown unit kind %r" % (u.kind,))
    return out


def param_count(units, height, width) -> int:
    return sum(int(np.prod(s)) for _, s, _, _ in param_layout(units, height, width))


def param_slices(units, height, width) -> Dict[str, slice]:
    out, off = {}, 0
    for name, shape, _, _ in param_layout(units, height, width):
        n = int(np.prod(shape))
        out[name] = slice(off, off + n)
        off += n
    return out


# --------------------------------------------------------------------------
# seeded draws
# --------------------------------------------------------------------------
def _rng(seed: int, stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([int(seed), int(stream)])))


def make_params(units, height, width, seed=MASTER_SEED, perturb=False) -> np.ndarray:
    """He-normal conv/linear weights (std = sqrt(2/fan_in)), gamma = 1, beta = 0, biases 0.

    With perturb=True biases, gamma and beta get small seeded offsets so that
    tests exercise their gradient paths at non-trivial values.
    """
    chunks = []
    for i, (_, shape, role, fan_in) in enumerate(param_layout(units, height, width)):
        g = _rng(seed, 1000 + i)
        n = int(np.prod(shape))
        if role in ("conv_w", "lin_w"):
            v = g.standard_normal(n) * math.sqrt(2.0 / fan_in)
        elif role == "gamma":
            v = np.ones(n) + (0.2 * g.standard_normal(n) if perturb else 0.0)
        else:  # beta, bias
            v = 0.1 * g.standard_normal(n) if perturb else np.zeros(n)
        chunks.append(v.astype(np.float32))
    return np.concatenate(chunks) if chunks else np.zeros(0, np.float32)


def make_images(batch, height, width, channels, seed=MASTER_SEED, pixels="gauss") -> np.ndarray:
    """NHWC fp32 images: uniform [0,1), or per-channel N(0.5, 0.25^2) clipped to [0,1]."""
    g = _rng(seed, 1)
    if pixels == "uniform":
        x = g.random((batch, height, width, channels))
    else:
        x = np.clip(0.5 + 0.25 * g.standard_normal((batch, height, width, channels)), 0.0, 1.0)
    return x.astype(np.float32)


def make_pixels_u8(batch, height, width, channels, seed=MASTER_SEED, pixels="gauss") -> np.ndarray:
    """NHWC uint8 images: the 8-bit pixels of a colour image (per-channel N(128, 64^2) clipped to 0..255, or uniform
    over 0..255); stand-ins for the 8-bit images of a dataset such as CIFAR."""
    g = _rng(seed, 5)
    if pixels == "uniform":
        return g.integers(0, 256, size=(batch, height, width, channels), dtype=np.uint8)
    x = np.rint(np.clip(128.0 + 64.0 * g.standard_normal((batch, height, width, channels)), 0.0, 255.0))
    return x.astype(np.uint8)


def make_labels(batch, classes, seed=MASTER_SEED) -> np.ndarray:
    return _rng(seed, 2).integers(0, classes, size=batch).astype(np.int32)


def make_batch(w: Workload, perturb=False):
    """(params fp32 flat, x fp32 NHWC, y int32) for a workload."""
    p = make_params(w.units, w.height, w.width, w.seed, perturb)
    x = make_images(w.batch, w.height, w.width, w.channels, w.seed, w.pixels)
    y = make_labels(w.batch, w.classes, w.seed)
    return p, x, y
