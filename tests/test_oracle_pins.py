"""Pins of the CPU oracle against things that are not the oracle: hand-worked
sequences, a from-scratch brute force of Eq. 1 (exact integers and fp32),
library routines for special cases, and the identities the paper states
(p = 0 is standard FPS, Sec. 3.2; prefix equivalence, Sec. 3.3; the ablation
remark of Sec. 4.7).  CPU only."""
import itertools
import os
from fractions import Fraction

import numpy as np
import pytest

from paper_2604_17720_amd import inputs

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _read_golden(name):
    idx = md = None
    with open(os.path.join(GOLD, name)) as f:
        for line in f:
            if line.startswith("idx:"):
                idx = np.array(line.split()[1:], dtype=np.int32)
            elif line.startswith("maxdist:"):
                md = np.array([float(t) for t in line.split()[1:]], dtype=np.float32)
    return idx, md


# --------------------------------------------------------------------------
# independent brute forces (no running-minimum array, nothing from oracle/)
# --------------------------------------------------------------------------
def brute_fps_int(pts, M, start):
    """Eq. 1 literally, in exact Python integers: for every pick recompute the
    minimum over ALL prior picks for every unsampled point; lowest index wins."""
    pts = [tuple(int(v) for v in p) for p in pts]
    sel = [start]
    vals = [None]
    while len(sel) < M:
        best, bestv = None, None
        for i, p in enumerate(pts):
            if i in sel:
                continue
            v = min(sum((a - b) ** 2 for a, b in zip(p, pts[q])) for q in sel)
            if bestv is None or v > bestv:
                best, bestv = i, v
        sel.append(best)
        vals.append(bestv)
    return sel, vals


def brute_fps_f32(xyz, M, start):
    """Eq. 1 from scratch in NumPy float32 (each op rounded, no FMA)."""
    x = np.asarray(xyz, dtype=np.float32)
    sel = [start]
    while len(sel) < M:
        q = x[sel]                                   # [S,3]
        d = x[:, None, :] - q[None, :, :]            # [N,S,3] fp32
        d2 = (d[..., 0] * d[..., 0] + d[..., 1] * d[..., 1]) + d[..., 2] * d[..., 2]
        assert d2.dtype == np.float32
        m = d2.min(axis=1)
        sel.append(int(np.argmax(m)))                # first maximum = lowest index
    return sel


# --------------------------------------------------------------------------
# O1: exact FPS
# --------------------------------------------------------------------------
@pytest.mark.parametrize("name,cloud", [
    ("collinear9.txt", lambda: inputs.lattice_line(9)),
    ("grid3x3.txt", lambda: inputs.lattice_grid(3, 3)),
])
def test_hand_worked(oracle, name, cloud):
    idx, md = _read_golden(name)
    got, gmd = oracle.fps_exact(cloud(), len(idx), 0, return_maxdist=True)
    assert got.tolist() == idx.tolist()
    assert np.array_equal(gmd, md)


def test_brute_force_exact_integers(oracle):
    rng = np.random.default_rng(7)
    for trial in range(120):
        n = int(rng.integers(2, 40))
        side = int(rng.integers(2, 6))             # small lattice => many ties
        cells = rng.permutation(side ** 3)[: min(n, side ** 3)]
        pts = np.stack([cells // (side * side), (cells // side) % side, cells % side], axis=1)
        n = pts.shape[0]
        start = int(rng.integers(0, n))
        sel, vals = brute_fps_int(pts, n, start)
        got, gmd = oracle.fps_exact(pts.astype(np.float32), n, start, return_maxdist=True)
        assert got.tolist() == sel, (trial, pts.tolist(), start)
        assert [int(v) for v in gmd[1:]] == vals[1:]


def test_brute_force_float32(oracle):
    for seed in range(40):
        n = 8 + 3 * seed
        x = inputs.uniform_cube(n, 5000 + seed)
        start = seed % n
        m = min(n, 24)
        assert oracle.fps_exact(x, m, start).tolist() == brute_fps_f32(x, m, start)


@pytest.mark.parametrize("threads", [1, 2, 3, 5, 8, 13])
def test_threaded_exact_fps(oracle, threads):
    """The all-cores entry (point chunks per iteration, chunk results merged in
    ascending chunk order) against the same pins as the single-thread loop:
    hand-worked sequences, the exact-integer brute force on tie-heavy lattices
    (chunks smaller than the thread count included), and equality with the
    single-thread run, indices and distance bits, on every kind of cloud."""
    for name, cloud in (("collinear9.txt", inputs.lattice_line(9)), ("grid3x3.txt", inputs.lattice_grid(3, 3))):
        idx, md = _read_golden(name)
        got, gmd = oracle.fps_exact_mt(cloud, len(idx), 0, threads, return_maxdist=True)
        assert got.tolist() == idx.tolist() and np.array_equal(gmd, md)
    rng = np.random.default_rng(70 + threads)
    for trial in range(25):
        side = int(rng.integers(2, 5))
        n = int(rng.integers(2, side ** 3 + 1))
        cells = rng.permutation(side ** 3)[:n]
        pts = np.stack([cells // (side * side), (cells // side) % side, cells % side], axis=1)
        start = int(rng.integers(0, n))
        sel, vals = brute_fps_int(pts, n, start)
        got, gmd = oracle.fps_exact_mt(pts.astype(np.float32), n, start, threads, return_maxdist=True)
        assert got.tolist() == sel and [int(v) for v in gmd[1:]] == vals[1:]
    clouds = [inputs.uniform_cube(1, 1), inputs.uniform_cube(7, 2), inputs.make_config(4, N=20011)[0],
              inputs.lattice_grid(17, 13, 5), np.repeat(inputs.lattice_grid(4, 4, 4), 3, axis=0),
              inputs.planes_and_clusters(5003, 9)]
    for x in clouds:
        n = x.shape[0]
        m, start = min(n, 400), n // 3
        a, amd = oracle.fps_exact(x, m, start, return_maxdist=True)
        b, bmd = oracle.fps_exact_mt(x, m, start, threads, return_maxdist=True)
        assert np.array_equal(a, b) and np.array_equal(amd.view(np.uint32), bmd.view(np.uint32))
    with pytest.raises(ValueError):
        oracle.fps_exact_mt(clouds[1], 3, 0, 0)


def test_each_pick_maximises_min_distance_in_float64(oracle):
    """Property from Eq. 1, checked in float64 so it does not depend on the
    fp32 rounding of either side: every pick attains the maximum of the
    minimum distance to the earlier picks, up to fp32 rounding."""
    x = inputs.make_config(2, B=1, N=300)[0]
    idx, md = oracle.fps_exact(x, 100, 0, return_maxdist=True)
    xd = x.astype(np.float64)
    for k in range(1, 100):
        d = ((xd[:, None, :] - xd[idx[:k]][None, :, :]) ** 2).sum(-1).min(axis=1)
        assert d[idx[k]] >= d.max() * (1 - 1e-5)
        assert abs(md[k] - d[idx[k]]) <= 1e-5 * d[idx[k]]


def test_m2_is_a_farthest_point_query(oracle):
    for seed in range(10):
        x = inputs.uniform_cube(500, 6000 + seed)
        d = x - x[3]
        d2 = (d[:, 0] * d[:, 0] + d[:, 1] * d[:, 1]) + d[:, 2] * d[:, 2]
        assert oracle.fps_exact(x, 2, 3).tolist() == [3, int(np.argmax(d2))]


def test_invariants(oracle):
    x = inputs.make_config(3, B=1, N=2000)[0]
    idx, md = oracle.fps_exact(x, 700, 5, return_maxdist=True)
    assert idx[0] == 5 and np.isinf(md[0])
    assert len(set(idx.tolist())) == 700
    assert np.all(np.diff(md[1:]) <= 0)            # greedy radius never grows
    # mirror an axis: squares are unchanged bit for bit
    xm = x.copy()
    xm[:, 1] = -xm[:, 1]
    assert np.array_equal(oracle.fps_exact(xm, 700, 5), idx)
    # permutation equivariance (continuous coordinates: no ties)
    perm = np.random.default_rng(1).permutation(x.shape[0])
    inv = np.empty_like(perm)
    inv[perm] = np.arange(perm.size)
    got = oracle.fps_exact(x[perm], 700, int(inv[5]))
    assert np.array_equal(perm[got], idx)
    # integer translation of a lattice is exact in fp32
    g = inputs.lattice_grid(5, 4, 3)
    a = oracle.fps_exact(g, 60, 0)
    b = oracle.fps_exact(g + np.float32([100, -37, 12]), 60, 0)
    assert np.array_equal(a, b)
    # M == N returns a permutation
    assert sorted(oracle.fps_exact(g, 60, 7).tolist()) == list(range(60))
    # identical points: every distance is 0, the argmax over all points returns index 0
    same = np.tile(np.float32([[0.25, -1.5, 3.0]]), (40, 1))
    i2, d2 = oracle.fps_exact(same, 9, 7, return_maxdist=True)
    assert i2.tolist() == [7] + [0] * 8 and np.all(d2[1:] == 0)
    # scaling by a power of two is exact: same picks, distances scaled by its square
    i3, d3 = oracle.fps_exact(x * np.float32(2.0 ** -40), 700, 5, return_maxdist=True)
    assert np.array_equal(i3, idx) and np.array_equal(d3[1:], md[1:] * np.float32(2.0 ** -80))


def test_batched_equals_per_cloud(oracle):
    x = inputs.make_config(2, B=3, N=200)
    got = oracle.fps_exact(x, 50, 0)
    for b in range(3):
        assert np.array_equal(got[b], oracle.fps_exact(x[b], 50, 0))


def test_invalid_arguments(oracle):
    x = inputs.uniform_cube(10, 1)
    for (m, s) in [(0, 0), (11, 0), (3, -1), (3, 10)]:
        with pytest.raises(ValueError):
            oracle.fps_exact(x, m, s)


# --------------------------------------------------------------------------
# O4: coverage radius
# --------------------------------------------------------------------------
def test_coverage_radius_against_scipy_and_2_approximation(oracle):
    from scipy.spatial.distance import cdist
    x = inputs.uniform_cube(400, 11)
    sel = oracle.fps_exact(x, 37, 0)
    ref = cdist(x.astype(np.float64), x[sel].astype(np.float64)).min(axis=1).max()
    assert abs(oracle.coverage_radius(x, sel) - ref) <= 1e-6 * ref
    g = inputs.lattice_grid(4, 4)
    assert oracle.coverage_radius(g, np.array([0], np.int32)) == pytest.approx(np.sqrt(18.0), abs=0)
    # greedy FPS is a 2-approximation of the optimal k-centre radius
    y = inputs.uniform_cube(12, 12)
    for m in (2, 3, 4):
        opt = min(oracle.coverage_radius(y, np.array(c, np.int32))
                  for c in itertools.combinations(range(12), m))
        assert oracle.coverage_radius(y, oracle.fps_exact(y, m, 0)) <= 2.0 * opt + 1e-12


# --------------------------------------------------------------------------
# O2: FPS-Prune
# --------------------------------------------------------------------------
def test_prune_sizes_golden(oracle):
    with open(os.path.join(GOLD, "prune_sizes.txt")) as f:
        rows = [list(map(int, l.split())) for l in f if l.strip() and not l.startswith("#")]
    for n, m, kn, kd, fl, nc, k, r in rows:
        assert oracle.prune_sizes(n, m, kn, kd, fl) == (nc, k, r)
        # rounding rule restated with exact rationals
        keep = Fraction(kn, kd)
        assert nc == (-(-n * keep // 1) if fl & 1 else n)
        assert k == (-(-m * keep // 1) if fl & 2 else m)


def _py_candidates(n, nc, start):
    c = sorted((start + (j * n) // nc) % n for j in range(nc))
    return c, c.index(start)


def test_candidates_closed_form(oracle):
    for n, nc, start in [(10, 10, 0), (10, 5, 0), (10, 3, 7), (1000, 334, 0), (1000, 334, 999),
                         (7, 5, 3), (200000, 50000, 0)]:
        c, pos = oracle.candidates(n, nc, start)
        pc, ppos = _py_candidates(n, nc, start)
        assert c.tolist() == pc and pos == ppos
        assert len(set(pc)) == nc                      # distinct
    c, _ = oracle.candidates(200000, 50000, 0)
    assert np.array_equal(c, 4 * np.arange(50000))     # keep = 1/4, start 0: every 4th point


def test_p0_is_standard_fps(oracle):
    """Sec. 3.2: p = 0 is the standard FPS."""
    for cloud, start in [(inputs.lattice_grid(4, 5, 2), 0), (inputs.lattice_grid(4, 5, 2), 17),
                         (inputs.make_config(4, N=1500)[0], 0), (inputs.make_config(4, N=1500)[0], 777)]:
        n = cloud.shape[0]
        for m in (1, 2, n // 3, n):
            for flags in (0, 1, 2, 3):
                assert np.array_equal(oracle.fps_prune(cloud, m, 1, 1, flags, start),
                                      oracle.fps_exact(cloud, m, start))


@pytest.mark.parametrize("kn,kd", [(1, 4), (1, 2), (3, 4), (2, 3)])
@pytest.mark.parametrize("flags", [1, 2, 3])
def test_prune_structure(oracle, kn, kd, flags):
    x = inputs.make_config(4, N=3001)[0]
    n, m, start = x.shape[0], 700, 13
    nc, k, r = oracle.prune_sizes(n, m, kn, kd, flags)
    got = oracle.fps_prune(x, m, kn, kd, flags, start).tolist()
    # FPS part: exact FPS of the gathered candidate cloud, mapped back
    cand, pos = _py_candidates(n, nc, start)
    loc = oracle.fps_exact(x[cand], k, pos)
    assert got[:k] == [cand[j] for j in loc]
    assert got[0] == start
    # fill part: strided ranks of the sorted complement, from the FULL cloud
    free = sorted(set(range(n)) - set(got[:k]))
    assert got[k:] == [free[(j * (n - k)) // r] for j in range(r)] if r else got[k:] == []
    assert len(set(got)) == m


def test_iteration_pruning_keeps_the_fps_prefix(oracle):
    """Sec. 4.7 remark: with candidate pruning fixed, iteration pruning leaves
    the leading (1-p) M1 samples identical to the full-loop run."""
    x = inputs.make_config(5, N=300000)[0][:6000]
    full = oracle.fps_prune(x, 1200, 1, 4, 1, 0)     # CP only
    both = oracle.fps_prune(x, 1200, 1, 4, 3, 0)     # CP + IP
    assert np.array_equal(full[:300], both[:300])
    ip = oracle.fps_prune(x, 1200, 1, 4, 2, 0)       # IP only == exact prefix
    assert np.array_equal(ip[:300], oracle.fps_exact(x, 300, 0))


# --------------------------------------------------------------------------
# O3: stage chain and FPS-Cache
# --------------------------------------------------------------------------
def _split(flat, ms):
    o = np.cumsum([0] + list(ms))
    return [flat[o[i]:o[i + 1]] for i in range(len(ms))]


@pytest.mark.parametrize("cloud", ["line", "grid", "c3", "c2"])
def test_prefix_equivalence_theorem(oracle, cloud):
    """Sec. 3.3: with no pruning, the independent per-layer FPS chain returns
    exactly the prefixes of layer 1 (ties included: lattice inputs)."""
    x = {"line": lambda: inputs.lattice_line(200),
         "grid": lambda: inputs.lattice_grid(12, 11, 2),
         "c3": lambda: inputs.make_config(3, B=1, N=3000)[0],
         "c2": lambda: inputs.make_config(2, B=1, N=1024)[0]}[cloud]()
    ms = (150, 40, 40, 9, 1)
    chain = oracle.fps_stages(x, ms, oracle.MODE_CHAIN)
    cached = oracle.fps_stages(x, ms, oracle.MODE_CACHED)
    assert np.array_equal(chain, cached)
    first = oracle.fps_exact(x, ms[0], 0)
    for part, m in zip(_split(cached, ms), ms):
        assert np.array_equal(part, first[:m])


def test_chain_is_composed_per_layer_fps(oracle):
    x = inputs.make_config(4, N=2500)[0]
    ms = (900, 300, 77)
    parts = _split(oracle.fps_stages(x, ms, oracle.MODE_CHAIN, 1, 2, 3, 4), ms)
    prev = oracle.fps_prune(x, ms[0], 1, 2, 3, 4)
    assert np.array_equal(parts[0], prev)
    for part, m in zip(parts[1:], ms[1:]):
        cur = prev[oracle.fps_exact(x[prev], m, 0)]
        assert np.array_equal(part, cur)
        prev = cur


def test_cached_on_pruned_layer(oracle):
    x = inputs.make_config(4, N=4000)[0]
    ms = (1000, 250, 60)                              # k = 250 at keep 1/4
    parts = _split(oracle.fps_stages(x, ms, oracle.MODE_CACHED, 1, 4, 3, 0), ms)
    p1 = oracle.fps_prune(x, 1000, 1, 4, 3, 0)
    cand, pos = _py_candidates(4000, 1000, 0)
    exact_on_candidates = np.array(cand, np.int32)[oracle.fps_exact(x[cand], 250, pos)]
    assert np.array_equal(parts[0], p1)
    assert np.array_equal(parts[1], exact_on_candidates)          # M_l <= k: pure FPS order
    assert np.array_equal(parts[2], exact_on_candidates[:60])
    # a chain over a pruned layer 1 re-samples among fill points too, so the
    # theorem does not apply to it: it only has to stay inside layer 1
    chain = _split(oracle.fps_stages(x, ms, oracle.MODE_CHAIN, 1, 4, 3, 0), ms)
    assert set(chain[1].tolist()) <= set(p1.tolist()) and chain[1][0] == 0
    assert set(chain[2].tolist()) <= set(chain[1].tolist())


def test_coverage_ratio_lower_bound(oracle):
    """Greedy FPS is a 2-approximation of the best coverage radius any set of
    the same size can reach, so radius(variant) / radius(exact) >= 0.5 for
    every pruned variant; a smaller ratio would be a bug.  (Upper bounds on
    the ratio are stated for the full-size benchmark clouds and are checked
    there: the radius is a worst-point statistic and is noisy at this size.)"""
    x = inputs.make_config(4, N=8000)[0]
    exact = oracle.fps_exact(x, 2000, 0)
    r_exact = oracle.coverage_radius(x, exact)
    for (kn, kd) in [(3, 4), (1, 2), (1, 4)]:
        for flags in (1, 2, 3):
            rho = oracle.coverage_radius(x, oracle.fps_prune(x, 2000, kn, kd, flags, 0)) / r_exact
            assert 0.5 <= rho < 4.0
    stages = oracle.fps_stages(x, (2000, 500), oracle.MODE_CACHED)
    assert oracle.coverage_radius(x, stages[2000:]) == oracle.coverage_radius(x, exact[:500])


# --------------------------------------------------------------------------
# seeded random select / fill (the literal "UniformSample" / "RandomSample" of
# Alg. 1, which the paper leaves unspecified)
# --------------------------------------------------------------------------
def test_perm_is_a_bijection_for_every_size_and_seed(oracle):
    for n in (1, 2, 3, 4, 5, 16, 17, 63, 64, 65, 1000, 4096, 4097, 20011):
        for seed in (0, 1, 2 ** 32, 2 ** 64 - 1, 0x0123456789ABCDEF):
            img = [oracle.perm(n, seed, j) for j in range(n)]
            assert sorted(img) == list(range(n)), (n, seed)


def test_perm_depends_on_the_seed_and_spreads_uniformly(oracle):
    n, nc, seeds = 60, 12, 600
    hits = np.zeros(n)
    first = set()
    for seed in range(seeds):
        img = [oracle.perm(n, seed, j) for j in range(nc)]
        first.add(tuple(img[:4]))
        hits[img] += 1
    assert len(first) > 0.9 * seeds                       # seeds give different draws
    expect = seeds * nc / n                               # each index equally likely
    assert np.all(np.abs(hits - expect) < 5 * np.sqrt(expect))
    # both 32-bit halves of the seed matter
    a = [oracle.perm(1000, 5, j) for j in range(50)]
    assert a != [oracle.perm(1000, 5 + 2 ** 32, j) for j in range(50)]
    assert a != [oracle.perm(1000, 6, j) for j in range(50)]


@pytest.mark.parametrize("kn,kd", [(1, 4), (2, 3)])
@pytest.mark.parametrize("flags", [1 | 4, 2 | 4, 3 | 4])
def test_random_prune_structure(oracle, kn, kd, flags):
    """Semantics of the random variant, rebuilt with Python sets from the
    permutation alone: candidates = images of the first N' arguments (with the
    seed point forced in), ascending; fill = first R images of a second
    permutation that FPS did not pick, in that order."""
    x = inputs.make_config(4, N=2003)[0]
    n, m, start, seed = 2003, 500, 77, 99
    nc, k, r = oracle.prune_sizes(n, m, kn, kd, flags)
    got = oracle.fps_prune(x, m, kn, kd, flags, start, seed).tolist()
    img = [oracle.perm(n, seed, j) for j in range(nc)]
    if start not in img:
        img[-1] = start
    cand = sorted(img)
    c2, pos = oracle.candidates_perm(n, nc, start, seed)
    assert c2.tolist() == cand and cand[pos] == start and len(set(cand)) == nc
    loc = oracle.fps_exact(x[cand], k, cand.index(start))
    assert got[:k] == [cand[j] for j in loc]
    picked = set(got[:k])
    fill = []
    j = 0
    while len(fill) < r:
        t = oracle.perm(n, seed ^ 0xD1B54A32D192ED03, j)
        if t not in picked:
            fill.append(t)
        j += 1
    assert got[k:] == fill
    assert len(set(got)) == m
    # keep = 1/1 is still standard FPS (Sec. 3.2), whatever the seed
    assert np.array_equal(oracle.fps_prune(x, m, 1, 1, flags, start, seed), oracle.fps_exact(x, m, start))
