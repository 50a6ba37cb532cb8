#!/usr/bin/env python3
"""Op-level ablation of the FlashFPS components on one MI355X.

For a synthetic benchmark cloud and its stage sizes, times the whole stage
chain with candidate pruning (CP), iteration pruning (IP) and FPS-Cache (FC)
switched on and off (the grid of Table 3 in the paper, Sec. 4.7) at the pruning
ratios of Sec. 4.2, and prints a Markdown table: wall-clock per chain,
speed-up over the all-off baseline (exact FPS at every layer), the number of
point-distance updates the run performs, and the reduction in updates.
Sec. 3.2 predicts ~1/(1-p)^2 fewer updates for CP+IP in layer 1.

    python -m paper_2604_17720_amd.ablation --config 4 [--reps 5]

Every number is measured on synthetic inputs of the paper's workload shapes;
the paper's own speed-ups (end-to-end network inference on other hardware) are
not comparable and are not reproduced here."""
from __future__ import annotations

import argparse
import itertools
import sys


def chain_updates(N, stages, keep, cp, ip, fc, prune_sizes):
    kn, kd = keep
    flags = (1 if cp else 0) | (2 if ip else 0)
    nc, k, _ = prune_sizes(N, stages[0], kn, kd, flags)
    upd = nc * (k - 1)
    if not fc:
        upd += sum(n * (m - 1) for n, m in zip(stages[:-1], stages[1:]))
    return upd


def main(argv=None):
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", type=int, default=4, choices=(3, 4, 5))
    ap.add_argument("--reps", type=int, default=5)
    args = ap.parse_args(argv)

    import torch

    from . import binding as fb
    from . import inputs

    spec = inputs.CONFIGS[args.config]
    x = torch.from_numpy(inputs.make_config(args.config)).cuda()
    B, N, stages = spec["B"], spec["N"], spec["stages"]
    ws = fb.make_workspace(B, N, stages[0])
    out = torch.empty((B, sum(stages)), dtype=torch.int32, device="cuda")

    def run(keep, cp, ip, fc):
        flags = (fb.FFPS_FLAG_CP if cp else 0) | (fb.FFPS_FLAG_IP if ip else 0)
        mode = fb.FFPS_MODE_CACHED if fc else fb.FFPS_MODE_CHAIN
        kn, kd = keep if flags else (1, 1)
        fb.ffps_cached_stages(x, stages, mode, kn, kd, flags, workspace=ws, out=out)

    def time_ms(keep, cp, ip, fc):
        run(keep, cp, ip, fc)
        torch.cuda.synchronize()
        best = float("inf")
        for _ in range(args.reps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            run(keep, cp, ip, fc)
            e1.record()
            torch.cuda.synchronize()
            best = min(best, e0.elapsed_time(e1))
        assert fb.ffps_last_status(ws) == 0
        return best

    base_ms = time_ms((1, 1), False, False, False)
    base_upd = B * chain_updates(N, stages, (1, 1), False, False, False, fb.ffps_prune_sizes)
    print(f"## Ablation, config {args.config}: B={B}, N={N}, stages {list(stages)}\n")
    print(f"Baseline (exact FPS at every layer): {base_ms:.3f} ms, {base_upd:.3e} updates.\n")
    print("| p | CP | IP | FC | ms | speed-up | updates | update reduction | 1/(1-p)^2 |")
    print("|---|---|---|---|---|---|---|---|---|")
    fc_ms = time_ms((1, 1), False, False, True)
    fc_upd = B * chain_updates(N, stages, (1, 1), False, False, True, fb.ffps_prune_sizes)
    print(f"| 0 |  |  | x | {fc_ms:.3f} | {base_ms / fc_ms:.2f} | {fc_upd:.3e} | "
          f"{base_upd / fc_upd:.2f} | 1.00 |")
    for keep in ((3, 4), (1, 2), (1, 4)):
        p = 1 - keep[0] / keep[1]
        for cp, ip, fc in itertools.product((True, False), repeat=3):
            if not (cp or ip):
                continue
            try:
                ms = time_ms(keep, cp, ip, fc)
            except fb.FlashFPSError as e:     # e.g. CP alone with k = M > N'
                print(f"| {p:.2f} | {'x' if cp else ''} | {'x' if ip else ''} | {'x' if fc else ''} | "
                      f"n/a ({fb.ffps_strerror(e.code)}) | | | | |")
                continue
            upd = B * chain_updates(N, stages, keep, cp, ip, fc, fb.ffps_prune_sizes)
            print(f"| {p:.2f} | {'x' if cp else ''} | {'x' if ip else ''} | {'x' if fc else ''} | "
                  f"{ms:.3f} | {base_ms / ms:.2f} | {upd:.3e} | {base_upd / upd:.2f} | "
                  f"{1 / (1 - p) ** 2:.2f} |")
    return 0


if __name__ == "__main__":
    sys.exit(main())
