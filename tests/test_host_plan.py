"""Host-side tests (no GPU): the C-ABI library loads and exports what the header declares; the planner's
byte counts, boundaries, budget check and argument validation."""
import ctypes
import os
import re

import pytest

from paper_2105_00619_amd import workloads as W
from paper_2105_00619_amd import binding
from paper_2105_00619_amd.binding import OptorchError, SeqPlan

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module", autouse=True)
def _built():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2105_00619_amd import build
        build.build(verbose=False)


def test_library_exports_every_declared_symbol():
    declared = set()
    for name in sorted(os.listdir(os.path.join(ROOT, "include"))):
        if not name.endswith(".h"):
            continue
        header = open(os.path.join(ROOT, "include", name)).read()
        header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
        declared |= set(re.findall(r"\b(optorch_\w+)\s*\(", header))
    assert declared and declared == set(binding.SYMBOLS)
    lib = ctypes.CDLL(binding.LIB_PATH)
    for name in declared:
        assert getattr(lib, name) is not None


def _plan(idx, **kw):
    return SeqPlan.from_workload(W.config(idx), **kw)


def test_param_counts_match_generator_layout():
    for idx in (1, 2, 3, 4, 5):
        w = W.config(idx)
        assert _plan(idx, activation_budget_bytes=0).param_count == W.param_count(w.units, w.height, w.width)


def test_large_image_config_plans_and_shrinks_with_k():
    # ResNet-18 on 16 images of 512 x 512 (the shape of the paper's memory experiment): 16 x the pixels of a
    # 32 x 32 batch of 256 per image; the plan must hold 64-bit sizes and k = 4 must cut the saved bytes
    w = W.config(6)
    assert (w.batch, w.height, w.width) == (16, 512, 512)
    p1 = _plan(6, k_segments=1)
    p4 = _plan(6)
    assert p1.param_count == W.param_count(w.units, w.height, w.width)
    # stem output alone: 16 x 512 x 512 x 64 fp32 = 1 GiB
    assert p1.planned_peak_saved_bytes > 16 * (1 << 30) and p1.act_arena_bytes >= p1.planned_peak_saved_bytes
    assert p4.planned_peak_saved_bytes < 0.5 * p1.planned_peak_saved_bytes
    assert p4.n_replay_launches > 0 and p1.n_replay_launches == 0


def _vgg_saved_bytes(z_only):
    # VGG-11-BN, fp32, batch 128, every activation stored: the input; per conv its pre-BN output Z, its post-ReLU
    # output A unless a max-pool follows (the pool's backward is done by the BatchNorm backward from Z and the pooled
    # gradient, so that A is read by nothing after the forward pass) or unless storage mode 1 rebuilds it, and the four
    # per-channel BN vectors; per pool its output (the last pool's output feeds only the head, which keeps the
    # flattened features and the loss gradient instead)
    b, e = 128, 4
    h, total, c = 32, b * 32 * 32 * 3 * e, 3
    widths = [64, "M", 128, "M", 256, 256, "M", 512, 512, "M", 512, 512, "M"]
    for i, wd in enumerate(widths):
        if wd == "M":
            h //= 2
            if i != len(widths) - 1:
                total += b * h * h * c * e
        else:
            c = wd
            keeps_a = not z_only and widths[i + 1] != "M"
            total += (2 if keeps_a else 1) * b * h * h * c * e + 4 * c * 4
    return total + b * 512 * 4 + b * 10 * 4  # head: features, loss gradient w.r.t. logits


def test_config2_all_stored_bytes_match_the_analytic_count():
    p = _plan(2, k_segments=1)
    assert p.planned_peak_saved_bytes == _vgg_saved_bytes(False) == 108838912
    assert p.n_replay_launches == 0


def test_storage_mode_1_keeps_z_only_analytic_count():
    # the same network with storage_mode 1: per conv only Z and the BN vectors are kept (A is rebuilt in backward where
    # something reads it: the three convolutions that feed another convolution), the pools' outputs and the input stay
    p0, p1 = _plan(2, k_segments=1), _plan(2, k_segments=1, storage_mode=1)
    assert p1.planned_peak_saved_bytes == _vgg_saved_bytes(True) < p0.planned_peak_saved_bytes
    assert p1.n_launches == p0.n_launches + 3  # one rebuilding pass per conv-BN-ReLU that feeds a convolution
    # ResNet-152 shape of config 5: the Z-only figure of the byte model (87.5 GiB all stored), plus the ReLU decisions
    # of the 50 block outputs as bits (a sixteenth of their 32.75 GiB), minus the last block's output, which backward
    # no longer reads (0.25 GiB)
    q = _plan(5, k_segments=1, storage_mode=1, activation_budget_bytes=0)
    blocks = 3 * 2.0 + 8 * 1.0 + 36 * 0.5 + 3 * 0.25  # GiB of block outputs: bf16, batch 4096
    assert abs(q.planned_peak_saved_bytes / 2 ** 30 - (87.5 + blocks / 16 - 0.25)) < 0.05
    # mode 2 writes and keeps every activation; in the 16-bit configurations modes 0 and 1 never write the activations
    # that a stride-1 convolution of the same unit rebuilds from z while it loads its operand, which in these networks
    # are most (3, 4) or all of those that mode 1 would otherwise rebuild in a pass of its own
    for idx in (3, 4):
        full = _plan(idx, activation_budget_bytes=0, storage_mode=2)
        a, bb = _plan(idx, activation_budget_bytes=0), _plan(idx, activation_budget_bytes=0, storage_mode=1)
        assert bb.planned_peak_saved_bytes <= a.planned_peak_saved_bytes < 0.95 * full.planned_peak_saved_bytes
        assert bb.act_arena_bytes <= a.act_arena_bytes < full.act_arena_bytes
        assert a.n_launches < full.n_launches
    a, bb = _plan(6, activation_budget_bytes=0), _plan(6, activation_budget_bytes=0, storage_mode=1)  # fp32: nothing folded
    assert bb.planned_peak_saved_bytes < 0.95 * a.planned_peak_saved_bytes and bb.act_arena_bytes < a.act_arena_bytes
    assert a.planned_peak_saved_bytes == _plan(6, activation_budget_bytes=0, storage_mode=2).planned_peak_saved_bytes


def test_automatic_choice_of_segments_and_storage_mode_under_a_budget():
    # k_segments 0 / storage_mode -1: fewest segments first, keeping activations before rebuilding them
    w = W.config(5)
    fixed = {k: _plan(5, k_segments=k, activation_budget_bytes=0).act_arena_bytes for k in (1, 2, 3, 4)}
    p = SeqPlan.from_workload(w, k_segments=0, storage_mode=-1)  # the configuration's 32 GiB
    # three segments do not fit with every remaining activation kept (fixed[3] is the least arena of any such plan), but do
    # once backward rebuilds them: taken before a fourth segment
    assert (p.k_segments, p.storage_mode) == (3, 1) and len(p.boundaries) == 2
    assert fixed[4] <= p.act_arena_bytes <= 32 * 2 ** 30 < fixed[3]
    p = SeqPlan.from_workload(w, k_segments=0, storage_mode=-1, activation_budget_bytes=0)
    assert (p.k_segments, p.storage_mode, p.act_arena_bytes) == (1, 0, fixed[1])
    # rebuilding activations is tried before a further segment
    v = W.config(2)
    a0 = _plan(2, k_segments=1, activation_budget_bytes=0).act_arena_bytes
    a1 = _plan(2, k_segments=1, storage_mode=1, activation_budget_bytes=0).act_arena_bytes
    p = SeqPlan.from_workload(v, k_segments=0, storage_mode=-1, activation_budget_bytes=(a0 + a1) // 2)
    assert (p.k_segments, p.storage_mode, p.act_arena_bytes) == (1, 1, a1)
    p = SeqPlan.from_workload(v, k_segments=0, storage_mode=0, activation_budget_bytes=(a0 + a1) // 2)
    assert p.k_segments > 1 and p.storage_mode == 0 and p.act_arena_bytes <= (a0 + a1) // 2
    p = SeqPlan.from_workload(v, k_segments=4, storage_mode=-1, activation_budget_bytes=0)
    assert (p.k_segments, p.storage_mode) == (4, 0)
    with pytest.raises(OptorchError) as e:
        SeqPlan.from_workload(v, k_segments=0, storage_mode=-1, activation_budget_bytes=2 ** 20)
    assert e.value.code == binding.E_BUDGET and "smallest" in str(e.value)
    with pytest.raises(OptorchError) as e:
        SeqPlan.from_workload(v, k_segments=0, boundaries=[3])
    assert e.value.code == binding.E_INVALID


def test_pool_is_computed_by_the_kernels_of_the_batchnorm_in_front_of_it():
    # VGG-11-BN has 5 max-pools, each behind a conv-BN-ReLU.  Backward: the BatchNorm backward always does the pool's
    # backward as well (5 launches fewer).  Forward: the BatchNorm apply does the pool too, unless the pool opens a
    # segment (then it is replayed from the segment's kept input and stays a kernel of its own).  All stored: 100
    # launches as separate kernels, 90 fused.  Equal-count k = 4 puts boundaries at units 3, 6, 9, all three of them pools.
    assert _plan(2, k_segments=1).n_launches == 90
    p = _plan(2, k_segments=4, plan_mode=0)
    assert p.boundaries == [3, 6, 9] and (p.n_launches, p.n_replay_launches) == (106, 13)
    # boundaries behind the pools instead: every pool is fused again, in the first pass and in the replay
    q = _plan(2, k_segments=4, boundaries=[4, 7, 10])
    assert (q.n_launches, q.n_replay_launches) == (101, 11)


def test_peak_shrinks_with_segments_and_plan_is_reproducible():
    p1, p4, p4b = _plan(2, k_segments=1), _plan(2, k_segments=4, plan_mode=0), _plan(2, k_segments=4, plan_mode=0)
    assert p4.boundaries == [3, 6, 9] == p4b.boundaries
    assert p4.planned_peak_saved_bytes < 0.6 * p1.planned_peak_saved_bytes
    assert (p4.act_arena_bytes, p4.planned_peak_saved_bytes) == (p4b.act_arena_bytes, p4b.planned_peak_saved_bytes)
    assert p4.n_replay_launches > 0 and p4.n_launches > p1.n_launches
    assert p4.act_arena_bytes >= p4.planned_peak_saved_bytes
    # the byte-aware plan is never worse than the equal-count plan
    pm = _plan(2, k_segments=4, plan_mode=1)
    assert pm.planned_peak_saved_bytes <= p4.planned_peak_saved_bytes
    # least recomputation within the least peak: the last segment (never replayed) takes every unit it can, so the
    # replay is shorter than under either other mode and nothing more is kept
    pt = _plan(2, k_segments=4, plan_mode=2)
    assert pt.boundaries == [2, 5, 7] == _plan(2).boundaries  # the benchmark configuration's own mode
    assert pt.planned_peak_saved_bytes <= pm.planned_peak_saved_bytes
    assert pt.n_replay_launches <= pm.n_replay_launches < p4.n_replay_launches
    for idx in (3, 4, 6):
        a, b, c = _plan(idx, plan_mode=0), _plan(idx, plan_mode=1), _plan(idx, plan_mode=2)
        assert c.planned_peak_saved_bytes <= a.planned_peak_saved_bytes
        assert c.n_replay_launches <= min(a.n_replay_launches, b.n_replay_launches)
    # under a budget the same mode spends the budget on a longer last segment
    t5, m5 = _plan(5, plan_mode=2), _plan(5, plan_mode=1)
    assert m5.act_arena_bytes < t5.act_arena_bytes <= 32 << 30 and t5.n_replay_launches < m5.n_replay_launches
    # 16-bit storage halves the activation bytes of the same plan (BN vectors and the fp32 head aside)
    ph = _plan(2, k_segments=1, precision=W.BF16)
    assert 0.49 < ph.planned_peak_saved_bytes / p1.planned_peak_saved_bytes < 0.51


def test_min_peak_plan_checkpoints_at_the_narrow_layer():
    # an hour-glass: wide - wide - narrow - wide - wide; one boundary (k = 2) belongs after the narrow layer
    units = [W.conv(3, 64), W.conv(64, 64), W.conv(64, 8), W.conv(8, 64), W.conv(64, 64), W.gap_linear_ce(64, 10)]
    p = SeqPlan(units, k_segments=2, precision=W.FP32, batch=32, height=32, width=32, channels=3, num_classes=10, plan_mode=1)
    assert p.boundaries == [3]
    eq = SeqPlan(units, k_segments=2, precision=W.FP32, batch=32, height=32, width=32, channels=3, num_classes=10, plan_mode=0)
    assert p.planned_peak_saved_bytes <= eq.planned_peak_saved_bytes
    ex = SeqPlan(units, k_segments=2, precision=W.FP32, batch=32, height=32, width=32, channels=3, num_classes=10, boundaries=[3])
    assert ex.planned_peak_saved_bytes == p.planned_peak_saved_bytes


def test_config5_budget_needs_the_byte_aware_plan():
    w = W.config(5)
    ok = SeqPlan.from_workload(w, plan_mode=1)  # min-peak plan, 32 GiB budget
    assert ok.act_arena_bytes <= 32 << 30
    # equal count needs 30 GiB where the byte-aware plan needs 20.5: under 24 GiB only the latter exists
    assert SeqPlan.from_workload(w, plan_mode=1, activation_budget_bytes=24 << 30).act_arena_bytes <= 24 << 30
    with pytest.raises(OptorchError) as e:
        SeqPlan.from_workload(w, plan_mode=0, activation_budget_bytes=24 << 30)
    assert e.value.code == binding.E_BUDGET
    with pytest.raises(OptorchError) as e:
        SeqPlan.from_workload(w, k_segments=1)  # all stored: far above the budget
    assert e.value.code == binding.E_BUDGET
    free = SeqPlan.from_workload(w, k_segments=1, activation_budget_bytes=0)
    assert free.planned_peak_saved_bytes > 3 * ok.planned_peak_saved_bytes


@pytest.mark.parametrize("units,kw", [
    ([W.conv(4, 8), W.gap_linear_ce(8, 10)], {}),                                   # cin does not match the image
    ([W.conv(3, 8)], {}),                                                            # no loss head
    ([W.gap_linear_ce(3, 10), W.conv(3, 8)], {}),                                    # head not last
    ([W.conv(3, 8), W.gap_linear_ce(8, 7)], {}),                                     # classes mismatch
    ([W.conv(3, 8, ksize=5, pad=2), W.gap_linear_ce(8, 10)], {}),                    # unsupported filter size
    ([W.conv(3, 8), W.gap_linear_ce(8, 10)], {"k_segments": 3}),                     # more segments than units
    ([W.conv(3, 8), W.conv(8, 8), W.gap_linear_ce(8, 10)], {"k_segments": 2, "boundaries": [0]}),  # bad boundary
    ([W.conv(3, 8), W.gap_linear_ce(8, 10)], {"precision": 7}),
    ([W.conv(3, 8), W.gap_linear_ce(8, 10)], {"storage_mode": 3}),
])
def test_invalid_arguments_are_rejected(units, kw):
    args = dict(k_segments=1, precision=W.FP32, batch=4, height=8, width=8, channels=3, num_classes=10)
    args.update(kw)
    with pytest.raises(OptorchError) as e:
        SeqPlan(units, **args)
    assert e.value.code == binding.E_INVALID and str(e.value)


def test_dataflow_argument_checks_need_no_gpu():
    lib = binding.load_library()
    assert [lib.optorch_encoded_words(z, 0) for z in (0, 1, 8, 9, 16, 17)] == [0, 1, 1, 2, 2, 0]
    assert [lib.optorch_encoded_words(z, 1) for z in (0, 1, 9, 10, 18, 19, 27, 28, 32, 33)] == [0, 1, 1, 2, 2, 3, 3, 4, 4, 0]
    buf = ctypes.create_string_buffer(64)
    addr = ctypes.addressof(buf)
    assert lib.optorch_encode(addr, 4, 8, 0, addr, None) == binding.E_INVALID
    assert b"1..16" in lib.optorch_dataflow_last_error()
    assert lib.optorch_encode(addr, -1, 8, 4, addr, None) == binding.E_INVALID
    assert lib.optorch_encode(None, 4, 8, 4, addr, None) == binding.E_INVALID
    assert lib.optorch_encode_lossless(addr, 4, 8, 33, addr, addr, None) == binding.E_INVALID
    assert lib.optorch_decode_normalized(addr, 4, 8, 4, 17, None, None, 0, addr, None) == binding.E_INVALID
    # an empty batch is a success that launches nothing
    assert lib.optorch_encode(None, 0, 8, 4, None, None) == binding.OK
    assert lib.optorch_decode_lossless(None, None, 4, 0, 4, None, None) == binding.OK


def test_planner_against_brute_force_on_small_networks():
    # every partition of two small networks, planned for real: plan mode 2 must find the least peak of saved bytes (its
    # byte model is not the schedule itself: 1 % of slack) with the least replay among the partitions that keep no
    # more than it does; plan mode 1 only promises a peak close to the least
    import itertools
    nets = [
        ([W.conv(3, 16), W.maxpool(), W.conv(16, 32), W.maxpool(), W.conv(32, 64), W.conv(64, 64), W.maxpool(),
          W.gap_linear_ce(64, 10)], W.FP32),
        ([W.conv(3, 16), W.basic_block(16, 16), W.basic_block(16, 32, 2), W.basic_block(32, 32), W.basic_block(32, 64, 2),
          W.bottleneck(64, 128, 2), W.gap_linear_ce(128, 10)], W.BF16),
    ]
    for units, precision in nets:
        kw = dict(batch=16, height=32, width=32, channels=3, num_classes=10, precision=precision)
        for k in (2, 3, 4):
            rows = []
            for b in itertools.combinations(range(1, len(units)), k - 1):
                p = SeqPlan(units, k_segments=k, boundaries=list(b), **kw)
                rows.append((p.planned_peak_saved_bytes, p.n_replay_launches))
            least = min(r[0] for r in rows)
            m1 = SeqPlan(units, k_segments=k, plan_mode=1, **kw)
            m2 = SeqPlan(units, k_segments=k, plan_mode=2, **kw)
            assert m2.planned_peak_saved_bytes <= 1.01 * least
            assert m2.n_replay_launches <= min(r[1] for r in rows if r[0] <= m2.planned_peak_saved_bytes)
            assert m1.planned_peak_saved_bytes <= 1.15 * least
