"""optorch_seq_step_static (the step for callers that cannot allocate: the activation arena is the library's static
device array) against optorch_seq_step, through the C ABI: identical bits, on two calls in a row of which the second is
the smaller one and so finds the first one's contents in the shared array."""
import numpy as np
import pytest

from paper_2105_00619_amd import workloads as W

pytestmark = pytest.mark.gpu

CASES = [
    # (units, classes, batch, H, W, precision, k, momentum)
    ([W.conv(3, 16), W.basic_block(16, 32, 2), W.bottleneck(32, 64, 1), W.maxpool(), W.conv(64, 64),
      W.gap_linear_ce(64, 7)], 7, 12, 20, 20, W.BF16, 3, 0.9),
    ([W.conv(3, 8), W.conv(8, 8, stride=2), W.gap_linear_ce(8, 5)], 5, 4, 9, 9, W.FP32, 2, 0.0),
]


def _run(tr, p, xd, yd, static):
    import torch
    tr.set_params(p)  # same weights, zero momentum, fresh loss scale
    gd = torch.full((tr.param_count,), float("nan"), dtype=torch.float32, device="cuda")
    outs = []
    for _ in range(2):  # the second step also exercises the momentum and the refreshed 16-bit copies
        r = tr.step(xd, yd, 0.05, gd, static_arena=static)
        outs.append((r, gd.cpu().numpy().copy(), tr.get_params(), tr.running_stats()))
    return outs


def test_static_arena_step_matches_step_on_two_calls_in_a_row():
    import torch
    from paper_2105_00619_amd.binding import SeqTrainer
    sizes = []
    for units, classes, b, h, w, precision, k, mom in CASES:  # the larger network first, then the smaller one
        p = W.make_params(units, h, w, 31, perturb=True)
        x = W.make_images(b, h, w, 3, 31)
        y = W.make_labels(b, classes, 31)
        xd, yd = torch.from_numpy(x).cuda(), torch.from_numpy(y).cuda()
        tr = SeqTrainer(units, k_segments=k, precision=precision, batch=b, height=h, width=w, channels=3,
                        num_classes=classes, momentum=mom)
        sizes.append(tr.act_arena_bytes)
        ref = _run(tr, p, xd, yd, static=False)
        got = _run(tr, p, xd, yd, static=True)
        for (r0, g0, w0, s0), (r1, g1, w1, s1) in zip(ref, got):
            assert r0 == r1, (r0, r1)  # loss, peaks, loss scale, skip flag
            assert not r0["skipped"] and np.isfinite(g0).all()
            assert np.array_equal(g0, g1) and np.array_equal(w0, w1) and np.array_equal(s0, s1)
        tr.close()
    assert sizes[1] < sizes[0]


def test_static_arena_step_rejects_a_plan_larger_than_the_static_arena():
    import torch
    from paper_2105_00619_amd.binding import E_BUDGET, OptorchError, SeqTrainer
    wl = W.config(3, batch=64)  # ResNet-18, bf16: about 80 MiB of activations
    tr = SeqTrainer.from_workload(wl)
    assert tr.act_arena_bytes > (32 << 20)
    p, x, y = W.make_batch(wl)
    tr.set_params(p)
    with pytest.raises(OptorchError) as ei:
        tr.step(torch.from_numpy(x).cuda(), torch.from_numpy(y).cuda(), 0.01, static_arena=True)
    assert ei.value.code == E_BUDGET and "static arena" in str(ei.value)
    assert np.array_equal(tr.get_params(), p)  # nothing ran
    tr.close()
