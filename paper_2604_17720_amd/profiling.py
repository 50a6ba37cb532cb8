#!/usr/bin/env python3
"""Profiling helpers for the FPS kernels on one MI355X.  Both sub-commands
print Markdown; the summaries under profiles/ are their output.

    python -m paper_2604_17720_amd.build --profile        (on the CPU, beforehand)
    python -m paper_2604_17720_amd.profiling phases        (on the GPU)

      Per-round phase breakdown of the register-resident kernels, measured
      inside the kernel by the profiling build (libflashfps_prof.so: the same
      sources with -DFFPS_PROFILE; workgroup 0's communication wave stamps the
      phases of every round with the 100 MHz wall clock and counts shader
      cycles inside the replay).

    python -m paper_2604_17720_amd.profiling summarize [--stats S.csv] [--trace T.csv] [--fetch F.csv --write W.csv]

      Tables from rocprofv3's CSV output: per-kernel time (--kernel-trace
      --stats) and HBM bytes per dispatch (--pmc FETCH_SIZE / --pmc WRITE_SIZE,
      one run each), the byte counters scaled by what they read for the
      256 MiB device copy of `bench.py --calibrate-copy` in the same run.
"""
from __future__ import annotations

import argparse
import collections
import csv
import os
import re
import sys

PHASES = ["loop top (outputs of the round before)", "wait for the workers' update of their last reports",
          "merge + publish", "gather (poll for all records)",
          "replay (count, compaction, wait for the workers, masks, settling)"]


def _phases(args) -> None:
    import torch

    from . import binding as fb
    from . import build as hip_build
    from . import inputs

    if not os.path.exists(hip_build.LIB_PROFILE):
        sys.exit("profiling build missing: run `python -m paper_2604_17720_amd.build --profile` first")
    fb.LIB_PATH = hip_build.LIB_PROFILE               # before the first call loads the library
    x4 = torch.from_numpy(inputs.make_config(4)).cuda()
    ws = fb.make_workspace(1, 200000, 50000)
    print("# Per-round phases of k_fps_grid, config 4 cloud (N = 200,000), from the profiling build\n")
    print("Command: `python -m paper_2604_17720_amd.profiling phases` after "
          "`python -m paper_2604_17720_amd.build --profile`.")
    print("Times are those of workgroup 0's communication wave (100 MHz wall clock), per round; cycles are "
          "shader cycles.\nThe workers apply the picks of the round before and make their next report while "
          "this wave is between `loop top` and the first barrier of the replay, so the wait at that barrier is "
          "what their path is longer by.\nThe instrumentation itself costs a few per cent (compare the kernel "
          "time below with bench.py's).\n")
    for picks, M in ((1, 4001), (16, 20000), (0, 50000)):
        var = fb.variant_with_picks(fb.FFPS_VARIANT_GRID, picks)
        fb.ffps_exact(x4, M, 0, var, workspace=ws)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        fb.ffps_exact(x4, M, 0, var, workspace=ws)
        e1.record()
        torch.cuda.synchronize()
        st = ws[:256].view(torch.int32).cpu().numpy().astype("int64")
        r = int(st[1])
        cap = "library default" if picks == 0 else str(picks)
        print(f"## picks per round capped at {cap}: M = {M}, {e0.elapsed_time(e1):.2f} ms, {r} rounds, "
              f"{(M - 1) / r:.1f} picks per round, {e0.elapsed_time(e1) * 1e3 / (M - 1):.3f} us per pick\n")
        print("| phase | ns per round |")
        print("|---|---|")
        for i, name in enumerate(PHASES):
            print(f"| {name} | {st[8 + i] * 10.0 / r:.0f} |")
        print(f"| sum | {sum(st[8:13]) * 10.0 / r:.0f} |")
        print()
        print(f"- polls per gather: {st[15] / r:.2f}")
        print(f"- inside the replay, shader cycles per round: bounds {st[24] / r:.0f}, counting {st[25] / r:.0f}, "
              f"compaction {st[26] / r:.0f}, work of the whole workgroup {st[27] / r:.0f}")
        print(f"- of which: own candidates back from LDS {st[32] / r:.0f}, first barrier (wait for the workers) {st[33] / r:.0f}, "
              f"this wave's share of the pairwise masks {st[34] / r:.0f}, second barrier {st[35] / r:.0f}, "
              f"settling the picks and handing them out {st[36] / r:.0f}")
        print(f"- per round: {st[28] / r:.1f} live candidates, {(M - 1) / r:.1f} picks, "
              f"{st[30] / r:.2f} rounds ended early by a lowered candidate")
        print(f"- rounds by number of live candidates: up to 64: {st[13]}, 65 to {3 * 64}: {st[14]}, "
              f"one pick at a time or none: {r - st[13] - st[14]}")
        print(f"- kernel: {st[16] * 0.01:.1f} us wall, {st[17] * 16 / (st[16] * 10.0):.3f} GHz shader clock\n")


def _short(name: str) -> str:
    name = name.replace("ffps::(anonymous namespace)::", "").replace("ffps::", "")
    return re.sub(r"distribution_elementwise_grid_stride_kernel<.*", "(torch uniform fill)", name)


def _summarize(args) -> None:
    if args.stats:
        print("| kernel | calls | total ms | average us | % | min us | max us |")
        print("|---|---|---|---|---|---|---|")
        for r in csv.DictReader(open(args.stats)):
            print(f"| `{_short(r['Name'])[:70]}` | {r['Calls']} | {int(r['TotalDurationNs']) / 1e6:.3f} | "
                  f"{float(r['AverageNs']) / 1e3:.1f} | {float(r['Percentage']):.2f} | "
                  f"{int(r['MinNs']) / 1e3:.1f} | {int(r['MaxNs']) / 1e3:.1f} |")
        print()
    if args.trace:
        # per kernel AND launch size: one instantiation serves clouds of several sizes
        d = collections.OrderedDict()
        for r in csv.DictReader(open(args.trace)):
            key = (_short(r["Kernel_Name"])[:70], int(r["Grid_Size_X"]) // max(int(r["Workgroup_Size_X"]), 1),
                   r["Workgroup_Size_X"])
            d.setdefault(key, []).append((int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3)
        total = sum(sum(v) for v in d.values())
        print("| kernel | workgroups x threads | calls | total ms | average us | % | min us | max us |")
        print("|---|---|---|---|---|---|---|---|")
        for k, v in sorted(d.items(), key=lambda kv: -sum(kv[1])):
            if sum(v) / total < 0.0005:
                continue
            print(f"| `{k[0]}` | {k[1]} x {k[2]} | {len(v)} | {sum(v) / 1e3:.3f} | {sum(v) / len(v):.1f} | "
                  f"{100 * sum(v) / total:.2f} | {min(v):.1f} | {max(v):.1f} |")
        print()
    if not (args.fetch and args.write):
        return

    def load(path):
        d = collections.OrderedDict()
        for row in csv.DictReader(open(path)):
            key = (_short(row["Kernel_Name"])[:60], row["Grid_Size"])
            d.setdefault(key, []).append(float(row["Counter_Value"]))
        return d

    f, w = load(args.fetch), load(args.write)
    copy = [k for k in f if "copyBuffer" in k[0] and max(f[k]) > 100000]
    kib = 256 * 1024.0
    fs = kib / max(f[copy[0]]) if copy else float("nan")
    wk = [k for k in w if "copyBuffer" in k[0] and max(w[k]) > 100000]
    wsc = kib / max(w[wk[0]]) if wk else float("nan")
    print(f"Calibration on the 256 MiB device copy: FETCH_SIZE reads {max(f[copy[0]]) if copy else 0:.2f} KiB "
          f"for 262144 KiB read (scale {fs:.3f}), WRITE_SIZE reads {max(w[wk[0]]) if wk else 0:.2f} KiB for "
          f"262144 KiB written (scale {wsc:.3f}).\n")
    print("| kernel | grid | calls | FETCH_SIZE KiB | bytes read | WRITE_SIZE KiB | bytes written | total |")
    print("|---|---|---|---|---|---|---|---|")
    for k, v in sorted(f.items(), key=lambda kv: -sum(kv[1]) / len(kv[1])):
        fv = sum(v) / len(v)
        wl = w.get(k, [0.0])
        wv = sum(wl) / len(wl)
        rd, wr = fv * fs * 1024, wv * wsc * 1024
        if rd + wr < 2e5:
            continue
        print(f"| `{k[0]}` | {k[1]} | {len(v)} | {fv:.1f} | {rd / 1e6:.1f} MB | {wv:.1f} | {wr / 1e6:.1f} MB | "
              f"{(rd + wr) / 1e6:.1f} MB |")
    if args.kernel:
        hits = [k for k in f if args.kernel in k[0]]
        if hits:
            k = max(hits, key=lambda kk: sum(f[kk]) / len(f[kk]))
            lo, hi = (int(t) if t else None for t in (args.launches or ":").split(":"))
            fl, wl = f[k][lo:hi], w.get(k, [0.0])[lo:hi]
            rd = sum(fl) / len(fl) * fs * 1024
            wr = sum(wl) / len(wl) * wsc * 1024
            print(f"\n`{k[0]}` (grid {k[1]}): FETCH_SIZE per launch {[round(v, 1) for v in f[k]]}, "
                  f"WRITE_SIZE per launch {[round(v, 1) for v in w.get(k, [])]} (KiB, dispatch order); "
                  f"mean over launches [{args.launches or ':'}]:\n")
            print(f"traffic_bytes_per_launch: {rd + wr:.0f}")
            print(f"read_bytes_per_launch: {rd:.0f}")
            print(f"written_bytes_per_launch: {wr:.0f}")


def main(argv=None) -> None:
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    sub = ap.add_subparsers(dest="cmd", required=True)
    sub.add_parser("phases")
    s = sub.add_parser("summarize")
    s.add_argument("--stats")
    s.add_argument("--trace", help="kernel trace CSV: table per kernel and launch size")
    s.add_argument("--fetch")
    s.add_argument("--write")
    s.add_argument("--kernel", help="kernel whose per-launch traffic is printed as `traffic_bytes_per_launch:`")
    s.add_argument("--launches", help="slice a:b of that kernel's launches (dispatch order) to average over")
    args = ap.parse_args(argv)
    {"phases": _phases, "summarize": _summarize}[args.cmd](args)


if __name__ == "__main__":
    main()
