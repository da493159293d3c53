"""GPU parity of the image data-flow path (encode / decode) against the CPU oracle, through the C ABI.

Integer results (encoded words, parities, decoded pixels) must be bit-exact.  The normalised decode computes one fused
multiply-add in fp32 and rounds once to the output type; against the float64 oracle that is half an ulp of the
output type: 2^-24 relative for fp32 (the fp32 rounding), 2^-9 for bf16 and 2^-12 for fp16, plus the fp32 rounding;
the tests allow twice that, and an absolute floor for results that cancel to near zero.
"""
import numpy as np
import pytest

from oracle import dataflow_oracle as D
from paper_2105_00619_amd import workloads as W
from tests.gpu_util import TOL, assert_parity, gpu_step, oracle_step

pytestmark = pytest.mark.gpu

REL = {W.FP32: 2.0 ** -23, W.BF16: 2.0 ** -8, W.FP16: 2.0 ** -11}


def _torch():
    import torch
    return torch


def _pixels(batch, n_pos, seed, pixels="uniform"):
    # n_pos need not factor into an image: a flat row of positions with 1 channel
    return W.make_pixels_u8(batch, 1, n_pos, 1, seed=seed, pixels=pixels).reshape(batch, n_pos)


def _u64(t):
    return t.cpu().numpy().view(np.uint64)


def _dev_words(words):
    torch = _torch()
    return torch.from_numpy(np.ascontiguousarray(words).view(np.int64)).cuda()


# (images per group, batch, positions): full and ragged groups, one and two words, several 2048-position tiles with a
# tail, positions that are not a multiple of 8 (per-position kernels), a single position, a single image
CASES = [(8, 16, 3072), (8, 19, 4104), (16, 35, 4104), (3, 7, 2056), (1, 2, 64), (9, 9, 2048), (12, 30, 5000),
         (5, 11, 1003), (16, 16, 1), (7, 3, 8), (2, 5, 6160)]


@pytest.mark.parametrize("z,batch,n_pos", CASES)
def test_encode_and_decode_match_oracle(z, batch, n_pos):
    from paper_2105_00619_amd import binding as B
    torch = _torch()
    X = _pixels(batch, n_pos, seed=1000 + z + batch)
    ref = D.encode_batch_words(X, z)
    a = B.encode(torch.from_numpy(X).cuda(), z)
    assert tuple(a.shape) == ref.shape
    assert np.array_equal(_u64(a), ref)
    # decode from the oracle's words (not from the GPU's own output)
    x = B.decode(_dev_words(ref), batch, n_pos, z)
    assert np.array_equal(x.cpu().numpy(), X)
    assert np.array_equal(x.cpu().numpy(), D.decode_batch_words(ref, z, batch))


def test_unaligned_buffers_take_the_per_position_kernels_with_the_same_result():
    from paper_2105_00619_amd import binding as B
    torch = _torch()
    z, batch, n_pos = 8, 10, 2048
    X = _pixels(batch, n_pos, seed=77)
    ref = D.encode_batch_words(X, z)
    raw = torch.zeros(batch * n_pos + 3, dtype=torch.uint8, device="cuda")
    xs = raw[3:].view(batch, n_pos)  # 3 bytes off any 8-byte boundary
    xs.copy_(torch.from_numpy(X).cuda())
    assert xs.data_ptr() % 8 != 0
    assert np.array_equal(_u64(B.encode(xs, z)), ref)
    out = torch.zeros(batch * n_pos + 5, dtype=torch.uint8, device="cuda")
    os_ = out[5:].view(batch, n_pos)
    B.decode(_dev_words(ref), batch, n_pos, z, out=os_)
    assert np.array_equal(os_.cpu().numpy(), X)
    assert int(out[:5].sum()) == 0  # nothing written in front of the buffer


def test_decoders_leave_missing_images_of_a_ragged_group_unwritten():
    from paper_2105_00619_amd import binding as B
    torch = _torch()
    z, batch, n_pos = 8, 11, 2048
    X = _pixels(batch, n_pos, seed=5)
    a = B.encode(torch.from_numpy(X).cuda(), z)
    buf = torch.full((16, n_pos), 171, dtype=torch.uint8, device="cuda")
    B.decode(a, batch, n_pos, z, out=buf[:batch])
    assert np.array_equal(buf[:batch].cpu().numpy(), X)
    assert bool((buf[batch:] == 171).all())


@pytest.mark.parametrize("precision", [W.FP32, W.BF16, W.FP16])
@pytest.mark.parametrize("z,batch,shape", [(8, 16, (32, 32, 3)), (16, 21, (9, 8, 3)), (4, 6, (5, 7, 3)), (8, 8, (16, 16, 1)),
                                           (3, 4, (4, 4, 16))])
def test_decode_normalized_matches_oracle(precision, z, batch, shape):
    from paper_2105_00619_amd import binding as B
    h, w, c = shape
    n_pos = h * w * c
    X = W.make_pixels_u8(batch, h, w, c, seed=31 + z).reshape(batch, n_pos)
    rng = np.random.default_rng(9)
    mean, std = rng.uniform(0.4, 0.55, c), rng.uniform(0.2, 0.3, c)
    scale = (1.0 / (255.0 * std)).astype(np.float32)
    shift = (-mean / std).astype(np.float32)
    words = D.encode_batch_words(X, z)
    ref = D.decode_normalized(words, z, batch, c, scale, shift)
    got = B.decode_normalized(_dev_words(words), batch, n_pos, z, c, scale, shift, precision).float().cpu().numpy()
    tol = REL[precision] * np.abs(ref) + 2.0 ** -22  # the sum's fp32 rounding is relative to pixel * scale, up to ~8
    assert np.all(np.abs(got - ref) <= tol), "worst %.3e" % np.max(np.abs(got - ref) - tol)


LL_CASES = [(1, 3, 64), (9, 20, 4096), (10, 10, 1028), (18, 40, 2052), (19, 19, 516), (27, 30, 1024), (28, 56, 260),
            (32, 70, 1536), (32, 5, 1001), (13, 13, 7)]


@pytest.mark.parametrize("z,batch,n_pos", LL_CASES)
def test_lossless_encode_and_decode_match_oracle(z, batch, n_pos):
    from paper_2105_00619_amd import binding as B
    torch = _torch()
    X = _pixels(batch, n_pos, seed=2000 + z)
    ref_a, ref_o = D.encode_lossless_batch_words(X, z)
    a, o = B.encode_lossless(torch.from_numpy(X).cuda(), z)
    assert np.array_equal(_u64(a), ref_a)
    assert np.array_equal(o.cpu().numpy().view(np.uint32), ref_o)
    x = B.decode_lossless(_dev_words(ref_a), torch.from_numpy(ref_o.view(np.int32)).cuda(), batch, n_pos, z)
    assert np.array_equal(x.cpu().numpy(), X)


def test_random_shapes_match_oracle():
    # seeded random (group size, batch, positions): tile tails, ragged groups and both kernel families in many mixes
    from paper_2105_00619_amd import binding as B
    torch = _torch()
    rng = np.random.default_rng(20210500619)
    for case in range(48):
        lossless = case % 3 == 2
        z = int(rng.integers(1, 33 if lossless else 17))
        batch = int(rng.integers(1, 3 * z + 2))
        n_pos = int(rng.choice([int(rng.integers(1, 64)), 8 * int(rng.integers(1, 400)), 4 * int(rng.integers(1, 600)),
                                int(rng.integers(1, 3000))]))
        X = rng.integers(0, 256, size=(batch, n_pos), dtype=np.uint8)
        xd = torch.from_numpy(X).cuda()
        what = "case %d: z=%d batch=%d n_pos=%d lossless=%d" % (case, z, batch, n_pos, lossless)
        if lossless:
            ref_a, ref_o = D.encode_lossless_batch_words(X, z)
            a, o = B.encode_lossless(xd, z)
            assert np.array_equal(_u64(a), ref_a) and np.array_equal(o.cpu().numpy().view(np.uint32), ref_o), what
            assert np.array_equal(B.decode_lossless(a, o, batch, n_pos, z).cpu().numpy(), X), what
        else:
            ref = D.encode_batch_words(X, z)
            a = B.encode(xd, z)
            assert np.array_equal(_u64(a), ref), what
            assert np.array_equal(B.decode(a, batch, n_pos, z).cpu().numpy(), X), what
            sc, sh = rng.uniform(0.001, 0.02, 1).astype(np.float32), rng.uniform(-2, 2, 1).astype(np.float32)
            got = B.decode_normalized(a, batch, n_pos, z, 1, sc, sh, W.FP32).cpu().numpy()
            want = D.decode_normalized(ref, z, batch, 1, sc, sh)
            assert np.all(np.abs(got - want) <= REL[W.FP32] * np.abs(want) + 2.0 ** -22), what


def test_empty_batch_and_argument_errors():
    from paper_2105_00619_amd import binding as B
    torch = _torch()
    x = torch.zeros((0, 64), dtype=torch.uint8, device="cuda")
    assert B.encode(x, 8).numel() == 0
    x = torch.zeros((4, 64), dtype=torch.uint8, device="cuda")
    for z in (0, 17, -1):
        with pytest.raises(B.OptorchError):
            B.encode(x, z)
    with pytest.raises(B.OptorchError):
        B.encode_lossless(x, 33)
    a = B.encode(x, 4)
    with pytest.raises(B.OptorchError):  # 3 channels do not divide 64 positions
        B.decode_normalized(a, 4, 64, 4, 3, [1, 1, 1], [0, 0, 0], W.FP32)


@pytest.mark.parametrize("z", [8, 16])
def test_benchmark_size_batch_sampled_against_oracle(z):
    # the largest batch of the benchmark configurations: 4096 images of 32 x 32 x 3
    from paper_2105_00619_amd import binding as B
    torch = _torch()
    batch, h, w, c = 4096, 32, 32, 3
    n_pos = h * w * c
    X = W.make_pixels_u8(batch, h, w, c, seed=8).reshape(batch, n_pos)
    xd = torch.from_numpy(X).cuda()
    a = B.encode(xd, z)
    got = _u64(a)  # [G, n_pos, words]
    rng = np.random.default_rng(z)
    for g in rng.choice(batch // z, 24, replace=False):
        cols = rng.choice(n_pos, 96, replace=False)
        ref = D.to_words(D.encode(X[g * z:(g + 1) * z][:, cols]), z // 8)
        assert np.array_equal(got[g][cols], ref)
    # properties that hold at any size: image i of a group is byte i of the words; the round trip is the identity
    view = got.reshape(batch // z, n_pos, z // 8).view(np.uint8).reshape(batch // z, n_pos, z)
    assert np.array_equal(view.transpose(0, 2, 1).reshape(batch, n_pos), X)
    assert bool((B.decode(a, batch, n_pos, z) == xd).all())


@pytest.mark.parametrize("precision", [W.FP32, W.BF16, W.FP16])
def test_step_on_an_encoded_batch_matches_oracle_and_the_plain_step(precision):
    from paper_2105_00619_amd import binding as B
    torch = _torch()
    units = [W.conv(3, 8), W.maxpool(), W.basic_block(8, 16, 2), W.gap_linear_ce(16, 5)]
    classes, b, h, w, c, z = 5, 12, 16, 16, 3, 8  # two groups, the second with 4 images
    p = W.make_params(units, h, w, 21, perturb=True)
    y = W.make_labels(b, classes, 21)
    X = W.make_pixels_u8(b, h, w, c, seed=21)
    scale = np.array([1 / (255 * 0.25), 1 / (255 * 0.24), 1 / (255 * 0.26)], dtype=np.float32)
    shift = np.array([-0.49 / 0.25, -0.48 / 0.24, -0.45 / 0.26], dtype=np.float32)
    words = D.encode_batch_words(X.reshape(b, -1), z)
    x_ref = D.decode_normalized(words, z, b, c, scale, shift).reshape(b, h, w, c)
    ls = 1024.0 if precision == W.FP16 else 1.0
    t = B.SeqTrainer(units, k_segments=2, precision=precision, batch=b, height=h, width=w, channels=c, num_classes=classes,
                     loss_scale_init=ls)
    t.set_params(p)
    yd = torch.from_numpy(y).cuda()
    gd = torch.zeros(t.param_count, dtype=torch.float32, device="cuda")
    r = t.step_encoded(_dev_words(words), z, scale, shift, yd, 0.0, gd)
    g_enc = gd.cpu().numpy().copy()
    loss, g = oracle_step(units, p, x_ref, y, precision, ls)
    assert not r["skipped"]
    assert abs(r["loss"] - loss) <= TOL[precision] * max(1.0, abs(loss))
    assert_parity(units, h, w, g_enc, g, TOL[precision], "encoded step")
    # the plain step on the decode layer's fp32 output sees the same input values: identical gradients
    xf = B.decode_normalized(_dev_words(words), b, h * w * c, z, c, scale, shift, W.FP32).view(b, h, w, c)
    t.set_params(p)
    r2 = t.step(xf, yd, 0.0, gd)
    assert r2["loss"] == r["loss"]
    assert np.array_equal(gd.cpu().numpy(), g_enc)
    # inference on the encoded batch = inference on the decode layer's output
    la = t.predict_encoded(_dev_words(words), z, scale, shift)
    lb = t.predict(xf)
    assert bool((la == lb).all()) and bool(torch.isfinite(la).all())
    t.close()
