#!/usr/bin/env python3
"""Benchmark of the FPS hot path on one MI355X.

One step = one pass of the whole path over the room-scale cloud (N = 200,000,
M1 = 50,000; stages 50000 -> 12500 -> 3125 -> 781), inputs resident in HBM:
  (a) exact FPS to M1                                  (ffps_exact)
  (b) FPS-Prune at p = 75 % + FPS-Cache prefixes       (ffps_cached_stages, CACHED)
  (c) FPS-Prune at p = 75 % + per-layer FPS chain      (ffps_cached_stages, CHAIN)
Prints ONE JSON line.  The metric is point-distance updates per second over
the whole step; the exact call (a), the dominant kernel, is also timed on its
own with events on the launch stream and priced against the HBM roofline at
20 algorithmic bytes per update."""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

N, STAGES = 200000, (50000, 12500, 3125, 781)
KEEP = (1, 4)
BYTES_PER_UPDATE = 20          # xyz 12 B + min-distance read 4 B + write 4 B
HBM_PEAK_GBS = 8000.0
# HBM bytes one launch of the dominant kernel really moves, from the hardware
# counters in profiles/k_fps_grid_config4_hbm_counters.md (FETCH_SIZE x 2.000 +
# WRITE_SIZE x 1.000, calibrated on a 256 MiB copy): exchange records only.
MEASURED_TRAFFIC_BYTES = 2.000 * 186856.25 * 1024 + 1.000 * 25891.39 * 1024


def updates_of_chain(sizes):
    return sum(n * (m - 1) for n, m in sizes)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-picks", type=int, default=50000,
                    help="picks of the oracle's bounded sample")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one 256 MiB device copy (reference for hardware byte counters)")
    ap.add_argument("--no-stream-probe", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU; --gpus above 1 is not supported "
                 "(the path has no multi-GPU part)")

    import numpy as np
    import torch

    import paper_2604_17720_amd.binding as fb
    from paper_2604_17720_amd import inputs

    torch.cuda.set_device(0)
    x_host = inputs.make_config(4)                     # [1, 200000, 3] fp32, seeded
    x = torch.from_numpy(x_host).cuda()
    M1 = STAGES[0]
    ws = fb.make_workspace(1, N, M1)
    out_exact = torch.empty((1, M1), dtype=torch.int32, device="cuda")
    out_stages = torch.empty((1, sum(STAGES)), dtype=torch.int32, device="cuda")
    flags = fb.FFPS_FLAG_CP | fb.FFPS_FLAG_IP
    nc, k, _ = fb.ffps_prune_sizes(N, M1, KEEP[0], KEEP[1], flags)

    upd_exact = N * (M1 - 1)
    upd_pruned = nc * (k - 1)
    upd_chain = upd_pruned + updates_of_chain(list(zip(STAGES[:-1], STAGES[1:])))
    upd_step = upd_exact + upd_pruned + upd_chain

    def step(events=None):
        if events:
            events[0].record()
        fb.ffps_exact(x, M1, 0, workspace=ws, out=out_exact)
        if events:
            events[1].record()
        fb.ffps_cached_stages(x, STAGES, fb.FFPS_MODE_CACHED, KEEP[0], KEEP[1], flags,
                              workspace=ws, out=out_stages)
        if events:
            events[2].record()
        fb.ffps_cached_stages(x, STAGES, fb.FFPS_MODE_CHAIN, KEEP[0], KEEP[1], flags,
                              workspace=ws, out=out_stages)
        if events:
            events[3].record()

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    assert fb.ffps_last_status(ws) == 0
    fb.ffps_exact(x, M1, 0, workspace=ws, out=out_exact)
    rounds_exact = fb.ffps_last_rounds(ws)

    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(evs[i])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    assert fb.ffps_last_status(ws) == 0

    ms_step = wall * 1e3 / args.steps
    ms_exact = sum(e[0].elapsed_time(e[1]) for e in evs) / args.steps
    ms_cached = sum(e[1].elapsed_time(e[2]) for e in evs) / args.steps
    ms_chain = sum(e[2].elapsed_time(e[3]) for e in evs) / args.steps
    achieved = upd_exact * BYTES_PER_UPDATE / (ms_exact * 1e-3) / 1e9

    if args.calibrate_copy:
        src = torch.empty(64 * 1024 * 1024, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        dst.copy_(src)                                  # reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()
        del src, dst

    result = {
        "metric": "point_distance_updates_per_s",
        "value": upd_step / (ms_step * 1e-3),
        "unit": "updates/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": "config 4: room-scale cloud N=200000, exact FPS to M=50000, "
                               "FPS-Prune p=75% (CP+IP) + FPS-Cache, and pruned per-layer chain; "
                               "stages 50000/12500/3125/781",
                   "N": N, "stages": list(STAGES), "keep": "1/4", "batch": 1},
        "exact_fps_ms": ms_exact,
        "exact_updates_per_s": upd_exact / (ms_exact * 1e-3),
        "us_per_pick_exact": ms_exact * 1e3 / (M1 - 1),
        "exchange_rounds_exact": rounds_exact,
        "picks_per_round_exact": (M1 - 1) / max(rounds_exact, 1),
        "flashfps_prune_cache_ms": ms_cached,
        "pruned_chain_ms": ms_chain,
        "speedup_prune_cache_vs_exact_layer1": ms_exact / ms_cached,
        "updates_per_step": upd_step,
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": MEASURED_TRAFFIC_BYTES,
                     "kernel": "k_fps_grid<6,3> (exact FPS, N=200000, M=50000)",
                     "algorithmic_bytes_per_launch": upd_exact * BYTES_PER_UPDATE,
                     "note": "points and min-distances stay in registers, so achieved is the "
                             "HBM-equivalent rate of a streaming loop, not bytes moved"},
    }

    # One plain grid barrier in the same launch shape (256 workgroups), and one
    # exchange round that delivers a single pick: the per-pick latency of the
    # multi-pick kernel is quoted against both.  The one-pick run uses the first
    # 100,000 points so that it is a different kernel instantiation and does not
    # mix into the profiler's average for the dominant kernel; the cost of a round
    # does not depend on the number of points per workgroup.
    result["grid_barrier_us"] = fb.ffps_barrier_probe(20000, workspace=ws)
    n_one, m_one = 100000, 4001
    x_one = x[:, :n_one].contiguous()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    one = fb.variant_with_picks(fb.FFPS_VARIANT_GRID, 1)
    fb.ffps_exact(x_one, m_one, 0, one, workspace=ws)
    e0.record()
    fb.ffps_exact(x_one, m_one, 0, one, workspace=ws)
    e1.record()
    torch.cuda.synchronize()
    result["us_per_round_one_pick"] = e0.elapsed_time(e1) * 1e3 / (m_one - 1)
    result["us_per_pick_over_grid_barrier"] = result["us_per_pick_exact"] / result["grid_barrier_us"]

    if not args.no_stream_probe:
        # Supplementary probe OUTSIDE the five configurations: a cloud too large for
        # on-chip residency (32 Mi uniform points), 64 picks, streamed from HBM.
        # One pick per pass shows the bandwidth the pass itself reaches.
        n_big, m_big = 1 << 25, 65
        g = torch.Generator(device="cuda")
        g.manual_seed(4242)
        xb = torch.rand((1, n_big, 3), generator=g, device="cuda", dtype=torch.float32)
        wsb = fb.make_workspace(1, n_big, m_big)
        ob = torch.empty((1, m_big), dtype=torch.int32, device="cuda")
        probe = {"workload": f"supplementary: N={n_big} uniform points, M={m_big}, "
                             "FFPS_VARIANT_STREAM", "bytes_per_pass": BYTES_PER_UPDATE * n_big}
        for name, picks in (("one_pick_per_pass", 1), ("default", 0)):
            var = fb.variant_with_picks(fb.FFPS_VARIANT_STREAM, picks)
            fb.ffps_exact(xb, m_big, 0, var, workspace=wsb, out=ob)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            fb.ffps_exact(xb, m_big, 0, var, workspace=wsb, out=ob)
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1)
            passes = fb.ffps_last_rounds(wsb)
            probe[name] = {
                "ms": ms, "passes": passes,
                "hbm_gbs_moved": BYTES_PER_UPDATE * n_big * passes / (ms * 1e-3) / 1e9,
                "hbm_gbs_algorithmic": BYTES_PER_UPDATE * n_big * (m_big - 1) / (ms * 1e-3) / 1e9,
            }
        probe["frac_of_peak_moved"] = probe["one_pick_per_pass"]["hbm_gbs_moved"] / HBM_PEAK_GBS
        result["stream_probe"] = probe
        del xb, wsb, ob

    if not args.no_cpu_baseline:
        import oracle
        oracle.build()
        m = min(args.cpu_picks, M1)
        t0 = time.perf_counter()
        ref = oracle.fps_exact(x_host[0], m, 0)
        dt = time.perf_counter() - t0
        got = out_exact.cpu().numpy()[0, :m]
        result["cpu_baseline"] = {
            "value": N * (m - 1) / dt, "unit": "updates/s", "cores": 1, "kind": "oracle",
            "sample": f"exact FPS on the same 200000-point cloud, first {m} of {M1} picks "
                      f"({dt:.1f} s, single thread)",
            "matches_gpu_prefix": bool(np.array_equal(ref, got)),
        }
    print(json.dumps(result))


if __name__ == "__main__":
    main()
