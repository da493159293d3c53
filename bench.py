#!/usr/bin/env python3
"""Benchmark of the checkpointed training step on one MI355X.

One "step" is one pass of the whole hot path over one synthetic batch: input cast, forward of the
non-last segments keeping only their inputs, forward of the last segment, per-segment replay +
backward, fused optimizer, read-back of loss and overflow flag.  Inputs are resident in HBM before
the timed region.  Prints ONE JSON line: images/sec, peak activation bytes, the roofline figure of
the dominant kernel class and the CPU oracle timed on the host cores on a bounded sample of the same
workload.  The default workload is the one the metric is quoted on: the ResNet-152-style network in bf16, batch 4096,
k = 7 segments under a 32 GiB activation budget (--config 5); every timed step returns its gradients.

Timing perturbs a step (a launch that carries its own start and stop event costs about 5 us of front-end
time; with all ~130-900 launches of a step timed that is a tenth of the step), so the per-class breakdown
comes from a short survey pass before the timed region, and inside the timed region only the launches of the
dominant class carry events, on every --timed-every-th step; the roofline figure is computed from those.
The events take the dispatch's own time stamps, so the durations are the kernels' own, as in a kernel trace.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK = {"hbm": 8000.0,  # GB/s
        "mfma_f32": 157.3, "mfma_bf16": 2500.0, "mfma_f16": 2500.0}  # TFLOP/s dense
MFMA_CLASSES = ("conv_fwd", "conv_dgrad", "conv_wgrad")  # 3x3 (and larger) convolutions: bound by the matrix cores
CONV_CLASSES = MFMA_CLASSES + ("conv1x1_fwd", "conv1x1_dgrad", "conv1x1_wgrad")
# 1x1 convolutions in the 16-bit modes are bound by HBM traffic (C_in * C_out / (C_in + C_out) FLOP per byte at best,
# 51 to 410 on the bottleneck networks, against a ridge of 2500 / 8 = 312); in fp32 mode (ridge 20) they are MFMA-bound.
# Forward and data gradient run the same kernels (the data gradient is the forward computation on dz with flipped
# taps / the transposed weights), which a kernel trace cannot tell apart: they form one group for the roofline figure.
GROUPS = {"conv_fwd": "conv_fwd+conv_dgrad", "conv_dgrad": "conv_fwd+conv_dgrad",
          "conv1x1_fwd": "conv1x1_fwd+conv1x1_dgrad", "conv1x1_dgrad": "conv1x1_fwd+conv1x1_dgrad"}
GROUP_KERNELS = {
    "conv_fwd+conv_dgrad": "conv3x3_patch_kernel, conv_igemm_kernel (+ splitk_epilogue_kernel), conv_fwd_smallc_kernel",
    "conv_wgrad": "conv_wgrad3x3_kernel, conv_wgrad_kernel, conv_wgrad_smallc_kernel (+ wgrad_reduce_kernel)",
    "conv1x1_fwd+conv1x1_dgrad": "conv1x1_ws_kernel, conv1x1_rows_kernel, conv1x1_large_kernel, conv1x1_kernel, conv_igemm_kernel (strided or few pixels)",
    "conv1x1_wgrad": "conv_wgrad_kernel (+ wgrad_reduce_kernel)",
}
DTYPE_NAME = {0: "f32", 1: "bf16", 2: "f16"}


def _cpu_model():
    try:
        for line in open("/proc/cpuinfo"):
            if line.lower().startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def _time_oracle(units, p, x, y, momentum, dtype, min_seconds, max_steps=64):
    import numpy as np
    from oracle import seqnet_oracle as O
    v = np.zeros_like(p, dtype=dtype)
    pp, xx = p.astype(dtype), x.astype(dtype)
    steps, t0 = 0, time.perf_counter()
    while True:
        O.train_step(units, pp, v, xx, y, 0.01, momentum, dtype)
        steps += 1
        dt = time.perf_counter() - t0
        if dt >= min_seconds or steps >= max_steps:
            return steps, dt


def cpu_baseline(config_index, sample_batch=None, min_seconds=6.0):
    """The oracle as it stands (numpy, all activations stored) on a bounded sample of the workload: whole training
    steps of the same network on `sample_batch` images (per-image cost does not depend on the batch).  Timed in its
    float32 instantiation on all host cores (`value`), on one thread, and in float64 (the precision the parity tests
    use) on all cores."""
    import numpy as np
    from paper_2105_00619_amd import workloads as W
    from threadpoolctl import threadpool_info, threadpool_limits
    full = W.config(config_index)
    if sample_batch is None:  # about 10-30 s of CPU work in total
        sample_batch = {1: 8, 2: 128, 3: 64, 4: 16, 5: 8, 6: 1}.get(config_index, 8)
    sample_batch = min(sample_batch, full.batch)
    sw = W.config(config_index, batch=sample_batch)
    p, x, y = W.make_batch(sw)
    cores = max([q.get("num_threads", 1) for q in threadpool_info()] or [1])
    s32, t32 = _time_oracle(sw.units, p, x, y, sw.momentum, np.float32, min_seconds)
    half = max(1, sample_batch // 2)
    s64, t64 = _time_oracle(sw.units, p[:], x[:half], y[:half], sw.momentum, np.float64, min_seconds / 2)
    one_batch = max(1, sample_batch // 4)
    s1w = W.config(config_index, batch=one_batch)
    p1, x1, y1 = W.make_batch(s1w)
    with threadpool_limits(limits=1):
        s1, t1 = _time_oracle(s1w.units, p1, x1, y1, s1w.momentum, np.float32, min_seconds / 2, max_steps=8)
    return {"value": s32 * sample_batch / t32, "unit": "images/sec", "cores": int(cores), "kind": "oracle",
            "sample": "%d float32 training steps of the same network on batch %d (%.1f s) on %d threads; the workload's "
                      "batch is %d" % (s32, sample_batch, t32, cores, full.batch),
            "dtype": "f32", "value_float64": s64 * half / t64, "value_one_thread": s1 * one_batch / t1,
            "one_thread_sample": "%d float32 steps on batch %d (%.1f s)" % (s1, one_batch, t1),
            "cpu_model": _cpu_model(), "host_cpus": os.cpu_count()}


def dataflow_cpu_baseline(z, n_pos, min_seconds=10.0):
    """The data-flow oracle as it stands (exact Python integers) on a bounded sample: whole groups of z images."""
    import numpy as np
    from oracle import dataflow_oracle as D
    from paper_2105_00619_amd import workloads as W
    X = W.make_pixels_u8(z, 32, 32, 3, seed=W.MASTER_SEED).reshape(z, -1)[:, :n_pos]
    groups = 0
    t0 = time.perf_counter()
    while True:
        words = D.to_words(D.encode(X), D.words_needed(z, 8))
        D.decode_normalized(words[None], z, z, 3, [1 / 255.0] * 3, [0.0] * 3)
        groups += 1
        dt = time.perf_counter() - t0
        if dt >= min_seconds:
            break
    return {"value": groups * z / dt, "unit": "images/sec", "cores": 1, "kind": "oracle",
            "sample": "%d groups of %d images of 32x32x3 encoded and decoded with normalisation in exact integers (%.1f s)"
                      % (groups, z, dt)}


def dataflow_main(args):
    """--path dataflow: one step = Encode of an epoch-sized set of 8-bit images in groups of 16, then the decode layer
    (Decode + normalisation + cast to bf16) over all of it; both kernels are bound by HBM traffic."""
    import numpy as np
    import torch
    from paper_2105_00619_amd import binding as B
    from paper_2105_00619_amd import workloads as W
    if not os.path.exists(B.LIB_PATH):
        import __graft_entry__
        __graft_entry__.build()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    batch, h, w, c, z = args.batch or 50000, 32, 32, 3, 16
    n_pos = h * w * c
    g = torch.Generator(device="cuda").manual_seed(W.MASTER_SEED)
    x = torch.randint(0, 256, (batch, n_pos), dtype=torch.uint8, device="cuda", generator=g)
    words = B.encoded_words(z)
    a = torch.empty((-(-batch // z), n_pos, words), dtype=torch.int64, device="cuda")
    out = torch.empty((batch, n_pos), dtype=torch.bfloat16, device="cuda")
    xb = torch.empty_like(x)
    scale, shift = [1 / (255 * 0.25)] * 3, [-0.5 / 0.25] * 3
    ops = {
        "encode_kernel": (lambda: B.encode(x, z, out=a), batch * n_pos * 2.0),
        "decode_kernel<bf16>": (lambda: B.decode_normalized(a, batch, n_pos, z, c, scale, shift, W.BF16, out=out), batch * n_pos * 3.0),
        "decode_kernel<u8>": (lambda: B.decode(a, batch, n_pos, z, out=xb), batch * n_pos * 2.0),
    }
    # Every kernel is timed inside the loop it belongs to (Encode, then a decoder, over buffers larger than the
    # last-level cache together), with events on the launch stream around each launch: back-to-back launches of one
    # kernel would find part of their input still cached from the previous launch.
    def timed_pair(first, second, steps):
        ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(steps)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for e in ev:
            e[0].record(); ops[first][0](); e[1].record(); ops[second][0](); e[2].record()
        torch.cuda.synchronize()
        wall = (time.perf_counter() - t0) / steps
        us = [sum(e[i].elapsed_time(e[i + 1]) for e in ev) * 1e3 / steps for i in (0, 1)]
        return wall, us

    for _ in range(args.warmup):
        for fn, _b in ops.values():
            fn()
    per_kernel = {}
    _, (_, us_u8) = timed_pair("encode_kernel", "decode_kernel<u8>", args.steps)
    assert bool((xb == x).all()), "decode(encode(x)) != x"
    _, (us_enc, us_dec) = timed_pair("encode_kernel", "decode_kernel<bf16>", args.steps)
    for name, us in (("encode_kernel", us_enc), ("decode_kernel<bf16>", us_dec), ("decode_kernel<u8>", us_u8)):
        nbytes = ops[name][1]
        per_kernel[name] = {"avg_launch_us": us, "bytes_per_launch": nbytes, "gb_per_s": nbytes / us / 1e3}
    # the timed region proper: the same steps without events
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        B.encode(x, z, out=a)
        B.decode_normalized(a, batch, n_pos, z, c, scale, shift, W.BF16, out=out)
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / args.steps
    dom = "decode_kernel<bf16>"
    from paper_2105_00619_amd import traffic as T
    workload = "dataflow_encode_decode_%dx32x32x3_z16" % batch
    measured = T.lookup(workload, dom)  # HBM bytes per launch from counters, while the kernels are the measured ones
    line = {
        "metric": "images/sec", "value": batch / dt, "unit": "images/sec", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": dt * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u8", "data": "synthetic",
        "config": {"workload": workload, "images": batch, "image": "32x32x3 uint8",
                   "images_per_group": z, "step": "Encode, then Decode + normalisation + cast to bf16"},
        "roofline": {"bound": "hbm", "achieved": per_kernel[dom]["gb_per_s"], "peak": PEAK["hbm"], "unit": "GB/s",
                     "frac": per_kernel[dom]["gb_per_s"] / PEAK["hbm"],
                     "traffic": measured["bytes_per_launch"] if measured else None, "kernel": dom,
                     "avg_launch_us": per_kernel[dom]["avg_launch_us"],
                     "algorithmic_bytes_per_launch": per_kernel[dom]["bytes_per_launch"],
                     "timing": "HIP events on the launch stream around each of %d launches inside the step loop" % args.steps},
        "kernels": per_kernel,
    }
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = dataflow_cpu_baseline(z, n_pos)
    print(json.dumps(line))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=5,
                    help="benchmark configuration 1..6 (default 5: ResNet-152-style bf16, batch 4096, k=7 under a 32 GiB "
                         "activation budget -- the workload the metric is quoted on; 2: VGG-11-BN fp32, 3: ResNet-18 bf16, "
                         "4: ResNet-50-style fp16, 6: ResNet-18 fp32 on 16 images of 512x512)")
    ap.add_argument("--k", type=int, default=None, help="override the number of segments (0: the fewest that fit the workload's activation budget)")
    ap.add_argument("--batch", type=int, default=None)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-batch", type=int, default=None, help="default: a batch that keeps the CPU leg to about 20 s")
    ap.add_argument("--survey-steps", type=int, default=2, help="untimed steps with every kernel class event-timed")
    ap.add_argument("--timed-every", type=int, default=4,
                    help="steps of the timed region whose dominant-class launches carry events: every n-th")
    ap.add_argument("--plan-mode", type=int, default=None,
                    help="override the workload's way of choosing segment boundaries: 0 equal unit count, 1 least peak "
                         "of saved bytes, 2 least recomputation within that peak or within the budget")
    ap.add_argument("--storage-mode", type=int, default=0,
                    help="0: keep Z and A of every conv-BN-ReLU (default); 1: keep Z only, rebuild A in backward; -1: 1 only if 0 does not fit the budget")
    ap.add_argument("--path", choices=("train", "dataflow"), default="train",
                    help="train: the checkpointed training step (default); dataflow: image Encode + decode layer")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: the step has no inter-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)

    if args.path == "dataflow":
        dataflow_main(args)
        return

    import numpy as np
    import torch
    from paper_2105_00619_amd import workloads as W
    from paper_2105_00619_amd.binding import SeqTrainer, LIB_PATH
    if not os.path.exists(LIB_PATH):
        import __graft_entry__
        __graft_entry__.build()
    assert torch.cuda.is_available(), "bench.py needs a GPU"

    wl = W.config(args.config, batch=args.batch)
    k = args.k if args.k is not None else wl.k_segments
    plan_mode = wl.plan_mode if args.plan_mode is None else args.plan_mode
    tr = SeqTrainer.from_workload(wl, k_segments=k, storage_mode=args.storage_mode, plan_mode=plan_mode)
    p, x, y = W.make_batch(wl)
    tr.set_params(p)
    xd, yd = torch.from_numpy(x).cuda(), torch.from_numpy(y).cuda()
    gd = torch.empty(tr.param_count, dtype=torch.float32, device="cuda")  # every step returns its gradients
    torch.cuda.synchronize()

    lr = 0.01
    for _ in range(args.warmup):
        r = tr.step(xd, yd, lr, gd)
    torch.cuda.synchronize()

    # survey pass (untimed): every class event-timed, to find the dominant one and report the breakdown
    tr.profile_select(None)
    tr.profile_enable(True)
    for _ in range(max(1, args.survey_steps)):
        tr.step(xd, yd, lr, gd)
    survey = tr.profile_read()
    entries = tr.profile_read_entries()
    tr.profile_enable(False)
    classes = {}
    for name, c in survey["classes"].items():
        if c["entries"] == 0:
            continue
        sec = c["gpu_ms"] * 1e-3
        classes[name] = {
            "launches_per_step": c["launches"] / survey["steps"], "ms_per_step": c["gpu_ms"] / survey["steps"],
            "avg_entry_us": c["gpu_ms"] * 1e3 / c["entries"],
            "gbps": c["bytes"] / sec / 1e9 if sec > 0 else None,
            "tflops": c["flops"] / sec / 1e12 if sec > 0 and c["flops"] > 0 else None,
        }
    groups = {}
    for name, c in classes.items():
        groups.setdefault(GROUPS.get(name, name), []).append(name)
    dom = max(groups, key=lambda g: sum(classes[n]["ms_per_step"] for n in groups[g]))
    members = groups[dom]

    # timed region: events only on the launches of the dominant group, on every n-th step
    every = max(1, args.timed_every)
    tr.profile_select(())
    tr.profile_enable(True)
    steps_timed = 0
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        if every > 1 or i == 0:
            tr.profile_select(members if i % every == 0 else ())
        steps_timed += 1 if i % every == 0 else 0
        r = tr.step(xd, yd, lr, gd)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    prof = tr.profile_read()
    tr.profile_enable(False)
    tr.profile_select(None)
    ms = dt / args.steps * 1e3
    dc = {k_: sum(prof["classes"][n][k_] for n in members) for k_ in ("gpu_ms", "flops", "bytes", "entries", "launches")}
    mfma_bound = members[0] in MFMA_CLASSES or (members[0] in CONV_CLASSES and wl.precision == 0)
    if mfma_bound:
        key = {0: "mfma_f32", 1: "mfma_bf16", 2: "mfma_f16"}[wl.precision]
        achieved = dc["flops"] / (dc["gpu_ms"] * 1e-3) / 1e12
        roof = {"bound": "mfma", "kernel": dom, "achieved": achieved, "peak": PEAK[key], "unit": "TFLOP/s",
                "frac": achieved / PEAK[key], "traffic": None}
    else:
        achieved = dc["bytes"] / (dc["gpu_ms"] * 1e-3) / 1e9
        roof = {"bound": "hbm", "kernel": dom, "achieved": achieved, "peak": PEAK["hbm"], "unit": "GB/s",
                "frac": achieved / PEAK["hbm"], "traffic": None}
    # HBM bytes per launch from rocprofv3 FETCH_SIZE / WRITE_SIZE runs, if they were taken on these very kernels
    from paper_2105_00619_amd import traffic as _traffic
    meas = _traffic.lookup(wl.name, dom)
    if meas is not None:  # per launch, like `achieved`
        roof["traffic"] = meas["bytes_per_step"] / max(1.0, dc["launches"] / steps_timed)
        roof["traffic_algorithmic"] = dc["bytes"] / max(1, dc["launches"])
    if mfma_bound:
        # `achieved` counts every launch's own algorithmic FLOPs, replayed forward launches included ("executed");
        # the model's own work (forward once, data gradient, weight gradient) over the same kernel time:
        replay = sum(e["flops"] for e in entries if e["kind"] in members and e["phase"] == 2) / survey["steps"]
        exe = sum(e["flops"] for e in entries if e["kind"] in members) / survey["steps"]
        roof["work"] = "executed (replayed forward launches count with their own FLOPs)"
        roof["achieved_model_work"] = achieved * (exe - replay) / exe if exe > 0 else None
        roof["frac_model_work"] = roof["achieved_model_work"] / roof["peak"] if exe > 0 else None
    roof["kernels"] = GROUP_KERNELS.get(dom, dom)
    roof["avg_launch_us"] = dc["gpu_ms"] * 1e3 / max(1, dc["launches"])
    roof["ms_per_step"] = dc["gpu_ms"] / steps_timed
    roof["launches_timed"] = int(dc["launches"])
    roof["steps_timed"] = steps_timed

    # convolution work per step: "model" = 3 x the forward pass (forward + data gradient + weight gradient of the
    # network itself), "executed" adds the replayed forward of the checkpointed segments
    fwd_flops = sum(e["flops"] for e in entries if e["kind"] in ("conv_fwd", "conv1x1_fwd") and e["phase"] in (0, 1)) / survey["steps"]
    exe_flops = sum(e["flops"] for e in entries if e["kind"] in CONV_CLASSES) / survey["steps"]
    peak_key = {0: "mfma_f32", 1: "mfma_bf16", 2: "mfma_f16"}[wl.precision]
    conv_work = {
        "model_gflop_per_step": 3 * fwd_flops / 1e9, "executed_gflop_per_step": exe_flops / 1e9,
        "model_tflops_over_step_time": 3 * fwd_flops / (ms * 1e-3) / 1e12,
        "executed_tflops_over_step_time": exe_flops / (ms * 1e-3) / 1e12,
        "model_frac_of_mfma_peak": 3 * fwd_flops / (ms * 1e-3) / 1e12 / PEAK[peak_key],
    }

    out = {
        "metric": "train images/sec at fixed HBM activation budget; peak activation bytes; MFMA util",
        "value": wl.batch / (ms * 1e-3), "unit": "images/sec", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": DTYPE_NAME[wl.precision], "data": "synthetic",
        "config": {"workload": wl.name, "batch": wl.batch, "k_segments": tr.k_segments, "storage_mode": tr.storage_mode, "image": "%dx%dx%d NHWC" % (wl.height, wl.width, wl.channels),
                   "boundaries": tr.boundaries, "plan_mode": plan_mode, "momentum": wl.momentum},
        "loss": r["loss"], "peak_saved_bytes": r["peak_saved_bytes"], "peak_arena_bytes": r["peak_arena_bytes"],
        "activation_budget_bytes": wl.budget_bytes, "launches_per_step": tr.n_launches,
        "replay_launches_per_step": tr.n_replay_launches,
        "roofline": roof, "conv_work": conv_work, "kernel_classes_survey": classes,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(args.config, args.cpu_sample_batch)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
