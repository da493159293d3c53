"""HBM traffic of the convolution kernels from rocprofv3 counters, kept beside the kernels it was measured on.

Two counter runs of the benchmark (`--pmc FETCH_SIZE`, then `--pmc WRITE_SIZE`; both report KiB per dispatch) and
the same two runs of `copy` below, a plain device copy of known size, whose readings calibrate the counters:

    rocprofv3 --pmc FETCH_SIZE --output-format csv -d out/f  -- python3 bench.py --no-cpu-baseline --steps 5 --warmup 2
    rocprofv3 --pmc WRITE_SIZE --output-format csv -d out/w  -- python3 bench.py --no-cpu-baseline --steps 5 --warmup 2
    rocprofv3 --pmc FETCH_SIZE --output-format csv -d out/cf -- python3 -m paper_2105_00619_amd.traffic copy
    rocprofv3 --pmc WRITE_SIZE --output-format csv -d out/cw -- python3 -m paper_2105_00619_amd.traffic copy
    python3 -m paper_2105_00619_amd.traffic ingest --workload vgg11_bn_fp32_k4 --steps 12 \
        --fetch out/f/*counter_collection.csv --write out/w/*counter_collection.csv \
        --cal-fetch out/cf/*counter_collection.csv --cal-write out/cw/*counter_collection.csv

The data-flow benchmark (`bench.py --path dataflow`) is counted the same way, with `--path dataflow` added to the two
bench.py commands and `ingest --workload dataflow_encode_decode_50000x32x32x3_z16 --per-launch ...`: its figures are
bytes per kernel launch.

`ingest` writes traffic.json next to this file together with a hash of the kernel sources; `lookup` (used by
bench.py) returns the figure only while that hash still matches, i.e. while the kernels are the ones measured.
(--steps is the number of training steps the benchmark run executed: warm-up + survey + timed.)
"""
import argparse
import csv
import glob
import hashlib
import json
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
STORE = os.path.join(HERE, "traffic.json")
COPY_MIB = 1024
COPY_REPS = 4

# kernel-name fragments of the groups bench.py reports
GROUP_KERNELS = {
    "conv_fwd+conv_dgrad": ("conv3x3_patch_kernel", "conv_igemm_kernel", "splitk_epilogue_kernel", "conv_fwd_smallc_kernel",
                            "conv_fwd_direct_kernel", "conv_dgrad_direct_kernel"),
    "conv1x1_fwd+conv1x1_dgrad": ("conv1x1_kernel", "conv1x1_large_kernel", "conv1x1_ws_kernel", "conv1x1_rows_kernel"),
    # one kernel family serves the 1x1 and the other weight gradients: counted together
    "conv_wgrad": ("conv_wgrad3x3_kernel", "conv_wgrad_kernel", "conv_wgrad_smallc_kernel", "wgrad_reduce_kernel",
                   "wave_reduce_kernel", "conv_wgrad_direct_kernel", "splitk_reduce_kernel"),
    "bn_apply": ("bn_apply_kernel", "bn_apply_pool_kernel"),
    # the reduction pass (colreduce_kernel in its BatchNorm-backward modes, template arguments 1, 3 and 4) and the apply pass
    "bn_bwd": ("bn_bwd_apply_kernel", "bn_bwd_finalize_kernel", "bn_bwd_pool", "ELi1EEEvNS_7RedArgsE", "ELi3EEEvNS_7RedArgsE",
               "ELi4EEEvNS_7RedArgsE", ", 1>(oseq::RedArgs)", ", 3>(oseq::RedArgs)", ", 4>(oseq::RedArgs)"),
}


# the data-flow benchmark's kernels (the bf16 instantiation appears under its mangled name in the counter files)
DATAFLOW_KERNELS = {
    "encode_kernel": ("encode_kernel<",),
    "decode_kernel<bf16>": ("decode_kernelILi1EDF16b", "decode_kernelILi2EDF16b", "decode_kernel<1, __bf16>", "decode_kernel<2, __bf16>"),
    "decode_kernel<u8>": ("decode_kernel<1, unsigned char>", "decode_kernel<2, unsigned char>"),
}


DATAFLOW_ONLY = ("k_dataflow.hip", "dataflow.cpp")          # sources of the data-flow kernels alone
SHARED = ("dev_common.h", "launch.h")                         # device helpers both kinds of kernels are built from


def source_hash(workload: str = "") -> str:
    """Hash of the sources a workload's kernels are built from: the data-flow files and the shared device helpers for
    the data-flow benchmark; everything but the data-flow files for a training workload."""
    dataflow = workload.startswith("dataflow")
    h = hashlib.sha1()
    for f in sorted(glob.glob(os.path.join(HERE, "csrc", "*"))):
        name = os.path.basename(f)
        if not name.endswith((".hip", ".h", ".cpp")):
            continue
        if dataflow and name not in DATAFLOW_ONLY + SHARED:
            continue
        if not dataflow and name in DATAFLOW_ONLY:
            continue
        h.update(name.encode())
        h.update(open(f, "rb").read())
    return h.hexdigest()


def lookup(workload: str, group: str):
    """Measured HBM bytes per training step of a kernel group, or None (never measured, or the kernels changed)."""
    if not os.path.exists(STORE):
        return None
    d = json.load(open(STORE))
    rec = d.get(workload)
    if not rec or rec.get("source_hash") != source_hash(workload):
        return None
    return rec.get("groups", {}).get(group)


def _sum_counter(path: str, counter: str, fragments, count=None) -> float:
    """Sum of a counter (KiB) over the dispatches whose kernel name contains one of the fragments (count: a list that
    receives the number of such dispatches)."""
    total, n = 0.0, 0
    for r in csv.DictReader(open(path)):
        if r["Counter_Name"] != counter:
            continue
        if any(f in r["Kernel_Name"] for f in fragments):
            total += float(r["Counter_Value"])
            n += 1
    if count is not None:
        count.append(n)
    return total


def copy() -> None:
    """A plain device-to-device copy of COPY_MIB MiB, COPY_REPS times (the calibration workload)."""
    import torch
    n = COPY_MIB * 1024 * 1024 // 4
    src = torch.empty(n, dtype=torch.float32, device="cuda")  # contents do not matter; no fill kernel in the trace
    dst = torch.empty_like(src)
    torch.cuda.synchronize()
    for _ in range(COPY_REPS):
        dst.copy_(src)
    torch.cuda.synchronize()
    print("copied %d MiB x %d" % (COPY_MIB, COPY_REPS))


def ingest(args) -> None:
    copy_frag = ("copyBuffer", "copy_kernel", "CopyKernel")  # the device-to-device copy, whatever the runtime names it
    want_kib = COPY_MIB * 1024.0 * COPY_REPS
    cal_f = _sum_counter(args.cal_fetch, "FETCH_SIZE", copy_frag)
    cal_w = _sum_counter(args.cal_write, "WRITE_SIZE", copy_frag)
    if cal_f <= 0 or cal_w <= 0:
        sys.exit("no copy kernel found in the calibration runs")
    ff, fw = want_kib / cal_f, want_kib / cal_w  # true KiB per counted KiB
    groups = {}
    if args.per_launch:
        for g, frags in DATAFLOW_KERNELS.items():
            nf, nw = [], []
            fetch = _sum_counter(args.fetch, "FETCH_SIZE", frags, nf) * ff * 1024.0
            write = _sum_counter(args.write, "WRITE_SIZE", frags, nw) * fw * 1024.0
            if not nf[0] or not nw[0]:
                sys.exit("no dispatch of %s in the counter files" % g)
            groups[g] = {"fetch_bytes_per_launch": fetch / nf[0], "write_bytes_per_launch": write / nw[0],
                         "bytes_per_launch": fetch / nf[0] + write / nw[0]}
    else:
        for g, frags in GROUP_KERNELS.items():
            fetch = _sum_counter(args.fetch, "FETCH_SIZE", frags) * ff * 1024.0 / args.steps
            write = _sum_counter(args.write, "WRITE_SIZE", frags) * fw * 1024.0 / args.steps
            groups[g] = {"fetch_bytes_per_step": fetch, "write_bytes_per_step": write, "bytes_per_step": fetch + write}
    d = json.load(open(STORE)) if os.path.exists(STORE) else {}
    d[args.workload] = {"source_hash": source_hash(args.workload), "steps_counted": args.steps,
                        "calibration": {"fetch_factor": ff, "write_factor": fw, "copy_mib": COPY_MIB, "reps": COPY_REPS},
                        "groups": groups}
    json.dump(d, open(STORE, "w"), indent=1, sort_keys=True)
    print(json.dumps(d[args.workload], indent=1))


def main() -> None:
    ap = argparse.ArgumentParser()
    sub = ap.add_subparsers(dest="cmd", required=True)
    sub.add_parser("copy")
    ing = sub.add_parser("ingest")
    for a in ("--fetch", "--write", "--cal-fetch", "--cal-write", "--workload"):
        ing.add_argument(a, required=True)
    ing.add_argument("--steps", type=int, default=1)
    ing.add_argument("--per-launch", action="store_true", help="the data-flow kernels: bytes per kernel launch")
    args = ap.parse_args()
    if args.cmd == "copy":
        copy()
    else:
        ingest(args)


if __name__ == "__main__":
    main()
