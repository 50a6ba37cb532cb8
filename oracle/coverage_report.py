#!/usr/bin/env python3
"""Coverage-radius ratios of the pruned and cached variants, from the oracle alone.

    python oracle/coverage_report.py > profiles/coverage_ratio_table.md

TEST INFRASTRUCTURE: calls only the CPU oracle (oracle/), SciPy and the seeded
input generators; nothing of the HIP path.

For a cloud P and a sample S the coverage radius R_P(S) is the largest distance
from a point of P to its nearest sample.  The table gives, for every benchmark
configuration, rho = R_P(S_variant) / R_P(S_exact) at equal |S| over the
original cloud (for a batch: the largest rho over its clouds):

  - layer 1 of FPS-Prune (Alg. 1) at keep ratios 3/4, 1/2, 1/4 (p = 25, 50,
    75 %), candidate pruning + iteration pruning, strided and random
    select/fill, against the bound stated before any measurement,
    1.5 / sqrt(1 - p);
  - the cached stages (Sec. 3.3) built on that layer 1: every stage with
    M_l <= k (k = the true FPS picks of layer 1) against 1.5; stages with
    M_l > k reach into the fill and are listed without a bound;
  - for the two large single clouds, candidate pruning alone and iteration
    pruning alone, to show which step of Alg. 1 costs how much.

Radii are computed with a k-d tree in float64 (SciPy) and checked against the
oracle's own brute-force coverage radius on the small configurations.
"""
from __future__ import annotations

import importlib.util
import math
import os
import sys

import numpy as np
from scipy.spatial import cKDTree

_HERE = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(_HERE)
sys.path.insert(0, _ROOT)
import oracle  # noqa: E402


def _inputs():
    # the seeded input generators, loaded as a plain module (no method arithmetic in it)
    spec = importlib.util.spec_from_file_location(
        "ffps_inputs", os.path.join(_ROOT, "paper_2604_17720_amd", "inputs.py"))
    mod = importlib.util.module_from_spec(spec)
    sys.modules["ffps_inputs"] = mod
    spec.loader.exec_module(mod)
    return mod


def radius(cloud: np.ndarray, sel: np.ndarray) -> float:
    d, _ = cKDTree(cloud[sel].astype(np.float64)).query(cloud.astype(np.float64), k=1, workers=-1)
    return float(d.max())


KEEPS = ((3, 4), (1, 2), (1, 4))


def main() -> None:
    inputs = _inputs()
    oracle.build()
    threads = oracle.host_threads()
    print("# Coverage-radius ratios of the pruned and cached variants (CPU oracle)\n")
    print("Command: `python oracle/coverage_report.py > profiles/coverage_ratio_table.md` (oracle, SciPy and the "
          "seeded inputs only).\n")
    print("rho = R_P(S_variant) / R_P(S_exact), same |S|, over the original cloud; for a batch the largest rho "
          "over its clouds.  Bounds were stated before any measurement: layer 1 <= 1.5 / sqrt(1 - p); cached "
          "stages with M_l <= k <= 1.5; rho >= 0.5 always.  A ratio above its bound is marked **over**.\n")

    # the k-d tree radius agrees with the oracle's brute force
    x1 = inputs.make_config(1)[0]
    s1 = oracle.fps_exact(x1, 512, 0)
    r_tree, r_brute = radius(x1, s1), oracle.coverage_radius(x1, s1)
    assert abs(r_tree - r_brute) <= 1e-5 * r_brute, (r_tree, r_brute)
    print(f"Check: config 1 exact sample, k-d tree radius {r_tree:.6f}, oracle brute force {r_brute:.6f}.\n")

    violations = []
    print("| config | mode | p | N' | k (true picks) | layer-1 rho | bound | cached stages: M_l (rho) | "
          "stages bound 1.5 |")
    print("|---|---|---|---|---|---|---|---|---|")
    for cfg in (1, 2, 3, 4, 5):
        spec = inputs.CONFIGS[cfg]
        clouds = inputs.make_config(cfg)
        B, N = clouds.shape[0], clouds.shape[1]
        Ms = list(spec["stages"])
        M1 = Ms[0]
        # exact reference: layer 1 and its prefixes (exact cached stages are prefixes, Sec. 3.3)
        exact = [oracle.fps_exact_mt(clouds[b], M1, 0, threads) for b in range(B)]
        r_exact = [[radius(clouds[b], exact[b][:m]) for m in Ms] for b in range(B)]
        for mode_name, extra in (("strided", 0), ("random", oracle.FLAG_PERM)):
            for kn, kd in KEEPS:
                flags = oracle.FLAG_CP | oracle.FLAG_IP | extra
                Np, k, _ = oracle.prune_sizes(N, M1, kn, kd, flags)
                bound = 1.5 / math.sqrt(kn / kd)
                rho1 = 0.0
                rho_st = [0.0] * len(Ms)
                for b in range(B):
                    out = oracle.fps_stages(clouds[b], Ms, oracle.MODE_CACHED, kn, kd, flags, 0, 1000 + b)
                    off = 0
                    for li, m in enumerate(Ms):
                        sel = out[off:off + m]
                        off += m
                        r = radius(clouds[b], sel) / r_exact[b][li]
                        if li == 0:
                            rho1 = max(rho1, r)
                        rho_st[li] = max(rho_st[li], r)
                p = 100 - 100 * kn // kd
                cells = []
                over_st = False
                for li in range(1, len(Ms)):
                    within = Ms[li] <= k
                    tag = "" if within else " (M_l > k, no bound)"
                    if within and rho_st[li] > 1.5:
                        over_st = True
                        violations.append(f"config {cfg}, {mode_name}, p={p} %, cached stage M={Ms[li]}: "
                                          f"rho {rho_st[li]:.3f} > 1.5")
                    cells.append(f"{Ms[li]} ({rho_st[li]:.3f}){tag}")
                over1 = rho1 > bound
                if over1:
                    violations.append(f"config {cfg}, {mode_name}, p={p} %, layer 1: rho {rho1:.3f} > {bound:.2f}")
                if min([rho1] + rho_st[1:]) < 0.5:
                    violations.append(f"config {cfg}, {mode_name}, p={p} %: a ratio below 0.5 (a bug)")
                print(f"| {cfg} (B={B}, N={N}) | {mode_name} | {p} % | {Np} | {k} | {rho1:.3f}"
                      f"{' **over**' if over1 else ''} | {bound:.2f} | {', '.join(cells) if cells else '-'} | "
                      f"{'**over**' if over_st else ('ok' if cells else '-')} |")
                sys.stdout.flush()

    # which step of Alg. 1 costs what: the two large single clouds, layer 1 only
    for cfg in (4, 5):
        x = inputs.make_config(cfg)[0]
        M1 = inputs.CONFIGS[cfg]["stages"][0]
        ex = oracle.fps_exact_mt(x, M1, 0, threads)
        r_ex = radius(x, ex)
        print(f"\n## Candidate pruning and iteration pruning on their own (config {cfg}, layer 1, strided)\n")
        print(f"R_P(S_exact) = {r_ex:.4f} at |S| = {M1}.\n")
        print("| p | candidate pruning only | iteration pruning only | both | bound |")
        print("|---|---|---|---|---|")
        for kn, kd in KEEPS:
            row = []
            for flags in (oracle.FLAG_CP, oracle.FLAG_IP, oracle.FLAG_CP | oracle.FLAG_IP):
                sel = oracle.fps_prune(x, M1, kn, kd, flags, 0, 0)
                row.append(radius(x, sel) / r_ex)
            print(f"| {100 - 100 * kn // kd} % | {row[0]:.3f} | {row[1]:.3f} | {row[2]:.3f} | "
                  f"{1.5 / math.sqrt(kn / kd):.2f} |")
            sys.stdout.flush()

    print("\n## Ratios above their bound\n")
    if violations:
        for v in violations:
            print(f"- {v}")
    else:
        print("None.")


if __name__ == "__main__":
    main()
