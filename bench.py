#!/usr/bin/env python3
"""Benchmark of the FPS hot path on one MI355X.

One step = one pass of the whole path over the room-scale cloud (N = 200,000,
M1 = 50,000; stages 50000 -> 12500 -> 3125 -> 781), inputs resident in HBM:
  (a) exact FPS to M1                                  (ffps_exact)
  (b) FPS-Prune at p = 75 % + FPS-Cache prefixes       (ffps_cached_stages, CACHED)
  (c) FPS-Prune at p = 75 % + per-layer FPS chain      (ffps_cached_stages, CHAIN)
Prints ONE JSON line.  `value` is the headline metric: point-distance updates
per second of exact FPS at N = 200,000, M = 50,000, i.e. N (M - 1) over the time
of call (a), taken with events on the launch stream inside the timed steps;
`ms_per_step` is the wall time of a whole step (a) + (b) + (c).

Roofline of the dominant kernel (k_fps_grid, call (a)): the cloud and its running
minimum distances stay in registers for the whole call, so no memory system
bounds it; what the hardware limits is the fp32 vector arithmetic of the
updates themselves.  An update is 3 subtractions, 3 multiplications, 2
additions and 1 minimum, each individually rounded: 9 operations that can
not be fused (the method fixes the rounding of each).  Peak for such code = half
the published 157.3 TFLOP/s fp32 vector rate, which counts a fused multiply-add
as two: 256 CUs x 4 SIMDs x 32 lanes per clock x 2.4 GHz = 78.6 T operations/s.
The rate that plain, unfused and unpacked fp32 instructions sustain on the
device is measured in the same run (`alu_probe`, the library's diagnostic
kernel) and reported beside it.
The HBM-equivalent rate (20 B per update over the same time: what a streaming
loop would have to move) is reported as an extra key, not as a roofline.

Supplementary probe outside the five configurations: a cloud too large for
on-chip residency (32 Mi points) on the streaming kernel, whose picks are
compared with the CPU oracle, priced against the 8 TB/s HBM peak."""
import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

N, STAGES = 200000, (50000, 12500, 3125, 781)
KEEP = (1, 4)
OPS_PER_UPDATE = 9             # 3 sub + 3 mul + 2 add + 1 min, none fused
BYTES_PER_UPDATE = 20          # xyz 12 B + min-distance read 4 B + write 4 B
HBM_PEAK_GBS = 8000.0
MI355X_CUS, MI355X_GHZ, SIMDS_PER_CU, LANES_PER_SIMD_CLOCK = 256, 2.4, 4, 32
ALU_PEAK_TOPS = MI355X_CUS * SIMDS_PER_CU * LANES_PER_SIMD_CLOCK * MI355X_GHZ / 1e3   # 78.6


def updates_of_chain(sizes):
    return sum(n * (m - 1) for n, m in sizes)


def traffic_from_profile(name):
    """HBM bytes per launch that the hardware counters saw, from the committed
    rocprofv3 summary (its `traffic_bytes_per_launch:` line), with the file it
    came from; (None, None) if there is no such summary."""
    path = os.path.join(ROOT, "profiles", name)
    try:
        m = re.search(r"^traffic_bytes_per_launch:\s*([0-9.eE+]+)", open(path).read(), re.M)
    except OSError:
        return None, None
    return (float(m.group(1)), "profiles/" + name) if m else (None, None)


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
    ap.add_argument("--no-per-config", action="store_true",
                    help="skip the per-configuration table (configs 1, 2, 3, 5)")
    ap.add_argument("--no-latency-probes", action="store_true",
                    help="skip the grid-barrier and one-pick-per-round reference measurements")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU; --gpus above 1 is not supported "
                 "(the path has no multi-GPU part)")

    import numpy as np
    import torch

    import paper_2604_17720_amd.binding as fb
    from paper_2604_17720_amd import inputs

    torch.cuda.set_device(0)
    props = torch.cuda.get_device_properties(0)
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
    achieved_tops = upd_exact * OPS_PER_UPDATE / (ms_exact * 1e-3) / 1e12
    traffic, traffic_src = traffic_from_profile("k_fps_grid_config4_hbm_counters.md")

    if args.calibrate_copy:
        src = torch.empty(64 * 1024 * 1024, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        dst.copy_(src)                                  # reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()
        del src, dst

    plan = fb.ffps_describe_plan(1, N, fb.FFPS_VARIANT_AUTO, props.multi_processor_count)
    result = {
        "metric": "point_distance_updates_per_s",
        "value": upd_exact / (ms_exact * 1e-3),
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
        "config": {"workload": "config 4: room-scale cloud N=200000; value = exact FPS to M=50000; a step "
                               "also runs FPS-Prune p=75% (CP+IP) + FPS-Cache and the pruned per-layer "
                               "chain over stages 50000/12500/3125/781",
                   "N": N, "stages": list(STAGES), "keep": "1/4", "batch": 1},
        "exact_fps_ms": ms_exact,
        "us_per_pick_exact": ms_exact * 1e3 / (M1 - 1),
        "exchange_rounds_exact": rounds_exact,
        "picks_per_round_exact": (M1 - 1) / max(rounds_exact, 1),
        "flashfps_prune_cache_ms": ms_cached,
        "pruned_chain_ms": ms_chain,
        "speedup_prune_cache_vs_exact_layer1": ms_exact / ms_cached,
        "whole_step": {"updates": upd_step, "updates_per_s": upd_step / (ms_step * 1e-3),
                       "note": "exact + pruned/cached + pruned chain over the wall time of a step"},
        "hbm_equivalent_gbs": upd_exact * BYTES_PER_UPDATE / (ms_exact * 1e-3) / 1e9,
        "device": {"name": props.name, "compute_units": props.multi_processor_count,
                   "clock_mhz": getattr(props, "clock_rate", 0) / 1e3 or None},
        "roofline": {"bound": "alu", "achieved": achieved_tops, "peak": ALU_PEAK_TOPS,
                     "unit": "TFLOP/s", "frac": achieved_tops / ALU_PEAK_TOPS,
                     "traffic": traffic, "traffic_source": traffic_src,
                     "kernel_time_profile": "profiles/k_fps_grid_bench_config4_kernel_stats.md (this command "
                                            "with --no-per-config: config 3's batch runs on the same "
                                            "instantiation and launch size)",
                     "kernel": f"k_fps_grid (exact FPS, N={N}, M={M1}; {plan[1]} workgroups, "
                               f"{plan[2]} reporting units)",
                     "ops_per_update": OPS_PER_UPDATE,
                     "algorithmic_ops_per_launch": upd_exact * OPS_PER_UPDATE,
                     "peak_derivation": "256 CUs x 4 SIMDs x 32 lanes per clock x 2.4 GHz = half the "
                                        "published 157.3 TFLOP/s, which counts a fused multiply-add as two "
                                        "(the method fixes the rounding of every operation, so none is fused)",
                     "note": "points and minimum distances stay in registers; `traffic` is what the "
                             "hardware counters saw for one launch (exchange records), from the "
                             "committed profile"},
    }

    if not args.no_latency_probes:
        # One plain grid barrier in the same launch shape (256 workgroups), and one
        # exchange round that delivers a single pick: the per-pick latency of the
        # multi-pick kernel is quoted against both.  The one-pick run uses the first
        # 100,000 points so that it is a different kernel instantiation and does not
        # mix into the profiler's average for the dominant kernel; the cost of a round
        # does not depend on the number of points per workgroup.
        result["grid_barrier_us"] = fb.ffps_barrier_probe(20000, workspace=ws)
        # what plain fp32 vector instructions sustain on this device (no memory traffic)
        result["alu_probe"] = {"unit": "T operations/s", "operations": "sub, mul, add, min on 16 values per lane",
                               "by_waves_per_cu": {str(wv): fb.ffps_alu_probe(wv, 20000, workspace=ws) / 1e12
                                                   for wv in (4, 8, 16, 32)}}
        result["roofline"]["sustained_by_plain_fp32"] = max(result["alu_probe"]["by_waves_per_cu"].values())
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
        result["us_per_pick_over_one_pick_round"] = (result["us_per_pick_exact"] /
                                                     result["us_per_round_one_pick"])
        del x_one

    def timed(fn, reps=5):
        """Mean time of fn() in ms over `reps` calls after one warm-up, by events."""
        fn()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(reps):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / reps

    if not args.no_per_config:
        # The other four configurations at their stated sizes: exact layer 1, the
        # exact chain (the baseline the paper calls FPS), and FPS-Prune p = 75 % +
        # FPS-Cache.  Their parity with the oracle is the tests' business.
        per = {}
        for c in (1, 2, 3, 5):
            spec = inputs.CONFIGS[c]
            B, n, st = spec["B"], spec["N"], spec["stages"]
            xc = torch.from_numpy(inputs.make_config(c)).cuda()
            wsc = fb.make_workspace(B, n, st[0])
            o1 = torch.empty((B, st[0]), dtype=torch.int32, device="cuda")
            oc = torch.empty((B, sum(st)), dtype=torch.int32, device="cuda")
            kernel, wg, units, clouds = fb.ffps_describe_plan(B, n, 0, props.multi_processor_count)
            t_exact = timed(lambda: fb.ffps_exact(xc, st[0], 0, workspace=wsc, out=o1))
            t_chain = timed(lambda: fb.ffps_cached_stages(xc, st, fb.FFPS_MODE_CHAIN, workspace=wsc, out=oc))
            t_flash = timed(lambda: fb.ffps_cached_stages(xc, st, fb.FFPS_MODE_CACHED, KEEP[0], KEEP[1],
                                                          flags, workspace=wsc, out=oc))
            assert fb.ffps_last_status(wsc) == 0
            upd = B * n * (st[0] - 1)
            per[f"config{c}"] = {
                "B": B, "N": n, "stages": list(st),
                "kernel": {1: "k_fps_wgm", 2: "k_fps_grid", 3: "k_fps_stream"}[kernel],
                "workgroups_per_cloud": wg, "units_per_cloud": units,
                "exact_layer1_ms": t_exact, "us_per_pick": t_exact * 1e3 / (st[0] - 1),
                "exact_updates_per_s": upd / (t_exact * 1e-3),
                "exact_chain_ms": t_chain, "prune75_cache_ms": t_flash,
                "speedup_flashfps_vs_exact_chain": t_chain / t_flash,
                "cache_bytes": 4 * st[0] * B,
            }
            del xc, wsc, o1, oc
        result["per_config"] = per

    stream_ref = None
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
        # per pass and point: xyz 12 B read, distance 4 B read (not in the first pass), 4 B written
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
            moved = n_big * (BYTES_PER_UPDATE * passes - 4)
            probe[name] = {
                "ms": ms, "passes": passes, "bytes_moved_algorithmic": moved,
                "hbm_gbs_moved": moved / (ms * 1e-3) / 1e9,
                "hbm_gbs_update_equivalent": BYTES_PER_UPDATE * n_big * (m_big - 1) / (ms * 1e-3) / 1e9,
                "picks": ob.cpu().numpy()[0].tolist(),
            }
        tr, tr_src = traffic_from_profile("k_fps_stream_probe_hbm_counters.md")
        one = probe["one_pick_per_pass"]
        probe["roofline"] = {"bound": "hbm", "achieved": one["hbm_gbs_moved"], "peak": HBM_PEAK_GBS,
                             "unit": "GB/s", "frac": one["hbm_gbs_moved"] / HBM_PEAK_GBS,
                             "traffic": tr, "traffic_source": tr_src,
                             "kernel": "k_fps_stream, one pick per pass (64 passes over 32 Mi points)"}
        # The streaming kernel forced onto the benchmark cloud, which is far too small
        # for it (a pass is latency-bound there): reported because the regime question
        # is asked of every configuration, not because it is the kernel to use.
        ob4 = torch.empty((1, M1), dtype=torch.int32, device="cuda")
        fb.ffps_exact(x, M1, 0, fb.FFPS_VARIANT_STREAM, workspace=ws, out=ob4)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        fb.ffps_exact(x, M1, 0, fb.FFPS_VARIANT_STREAM, workspace=ws, out=ob4)
        e1.record()
        torch.cuda.synchronize()
        ms4, passes4 = e0.elapsed_time(e1), fb.ffps_last_rounds(ws)
        probe["config4_forced_onto_stream"] = {
            "ms": ms4, "passes": passes4, "picks_per_pass": (M1 - 1) / passes4,
            "hbm_gbs_moved": N * (BYTES_PER_UPDATE * passes4 - 4) / (ms4 * 1e-3) / 1e9,
            "matches_register_resident_kernel": bool(torch.equal(ob4, out_exact)),
        }
        del ob4
        result["stream_probe"] = probe
        stream_ref = (xb.cpu().numpy()[0], m_big)
        del xb, wsb, ob

    if not args.no_cpu_baseline:
        import oracle
        oracle.build()
        m = min(args.cpu_picks, M1)
        threads = oracle.host_threads()
        t0 = time.perf_counter()
        ref_mt = oracle.fps_exact_mt(x_host[0], m, 0, threads)
        dt_mt = time.perf_counter() - t0
        m1 = m
        t0 = time.perf_counter()
        ref = oracle.fps_exact(x_host[0], m1, 0)
        dt = time.perf_counter() - t0
        got = out_exact.cpu().numpy()[0, :m]
        result["cpu_baseline"] = {
            "value": N * (m - 1) / dt_mt, "unit": "updates/s", "cores": threads, "kind": "oracle",
            "sample": f"exact FPS on the same 200000-point cloud, first {m} of {M1} picks on "
                      f"{threads} threads ({dt_mt:.1f} s); single thread: first {m1} picks ({dt:.1f} s)",
            "single_thread_value": N * (m1 - 1) / dt,
            "host_cpu_count": os.cpu_count(),
            "host_cpus_usable": len(os.sched_getaffinity(0)),
            "matches_gpu_prefix": bool(np.array_equal(ref_mt, got) and np.array_equal(ref, got[:m1])),
        }
        if stream_ref is not None:
            xs, ms_ = stream_ref
            t0 = time.perf_counter()
            want = oracle.fps_exact_mt(xs, ms_, 0, threads).tolist()
            p = result["stream_probe"]
            p["matches_oracle"] = bool(p["one_pick_per_pass"]["picks"] == want and
                                       p["default"]["picks"] == want)
            p["oracle_seconds"] = time.perf_counter() - t0
    if "stream_probe" in result:
        for name in ("one_pick_per_pass", "default"):
            del result["stream_probe"][name]["picks"]
    print(json.dumps(result))
    sys.stdout.flush()
    # release device memory in an orderly way before the interpreter tears down
    del x, ws, out_exact, out_stages, evs
    torch.cuda.synchronize()
    torch.cuda.empty_cache()


if __name__ == "__main__":
    main()
