"""Step time and activation memory as a function of the number of segments k (the method's trade-off).

    python3 -m paper_2105_00619_amd.sweep_k --config 2 [--plan-mode 0|1|2] [--steps 20]

Prints one line per k: ms per step, planned peak of saved activations, arena high-water mark, and both relative
to k = 1 (all activations stored, no recomputation).
"""
import argparse
import time


def main() -> None:
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", type=int, default=2)
    ap.add_argument("--plan-mode", type=int, default=None, help="0 equal count, 1 least peak bytes, 2 least recomputation within that peak (default: the config's)")
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--batch", type=int, default=None)
    ap.add_argument("--ks", type=str, default=None, help="comma-separated k values (default 1..number of units)")
    args = ap.parse_args()

    import torch
    from paper_2105_00619_amd import workloads as W
    from paper_2105_00619_amd.binding import SeqTrainer

    wl = W.config(args.config, batch=args.batch)
    p, x, y = W.make_batch(wl)
    xd, yd = torch.from_numpy(x).cuda(), torch.from_numpy(y).cuda()
    n_units = len(wl.units)
    ks = [int(v) for v in args.ks.split(",")] if args.ks else list(range(1, n_units))
    mode = wl.plan_mode if args.plan_mode is None else args.plan_mode
    base = None
    print("# %s, batch %d, plan mode %d" % (wl.name, wl.batch, mode))
    print("# k  boundaries  ms/step  saved MiB  arena MiB  time/time(k=1)  saved/saved(k=1)")
    for k in ks:
        tr = SeqTrainer.from_workload(wl, k_segments=k, plan_mode=mode, activation_budget_bytes=0)
        tr.set_params(p)
        for _ in range(args.warmup):
            r = tr.step(xd, yd, 0.01)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            r = tr.step(xd, yd, 0.01)
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) / args.steps * 1e3
        if base is None:
            base = (ms, r["peak_saved_bytes"])
        print("%3d  %-28s %8.3f %10.1f %10.1f %8.3f %8.3f" % (
            k, tr.boundaries, ms, r["peak_saved_bytes"] / 2**20, r["peak_arena_bytes"] / 2**20, ms / base[0],
            r["peak_saved_bytes"] / base[1]), flush=True)
        tr.close()


if __name__ == "__main__":
    main()
