"""The protocol by which the grid kernel overlaps its rounds
(paper_2604_17720_amd/csrc/fps_grid.hip), written out in NumPy and checked
against the oracle's exact FPS (Eq. 1) on small clouds.

A statement about the protocol, not about the kernels (those are compared with
the oracle element by element in the GPU tests).  Every reporting unit keeps the
three best points of each of its waves as of ONE ROUND EARLIER; their values are
brought up to date exactly, the waves' bounds (fourth values) are the old ones.
A round may pick only candidates above the largest bound, its first pick
included, and if none is, it picks nothing and the next round starts from exact
reports.  The picks must be those of Eq. 1, in order, whatever the layout."""
import numpy as np
import pytest

from paper_2604_17720_amd import inputs

f32 = np.float32


def sqdist(p, q):
    d = p - q
    return ((d[..., 0] * d[..., 0]) + (d[..., 1] * d[..., 1])) + (d[..., 2] * d[..., 2])   # fp32, this order


def wave_tops(m, members, keep):
    """Per wave: its `keep` best points (value descending, index ascending) and the next value."""
    vals = np.where(members >= 0, m[np.maximum(members, 0)], f32(-1))
    order = np.lexsort((members, -vals), axis=1)[:, :keep + 1]
    return np.take_along_axis(vals, order, 1), np.take_along_axis(members, order, 1)


def overlapped_fps(x, M, units, waves, keep=3, max_live=192):
    n = len(x)
    # point i: unit i mod units, wave (i div units) mod waves
    ids = np.arange(n)
    grp = (ids % units) * waves + (ids // units) % waves
    width = max(np.bincount(grp, minlength=units * waves))
    members = np.full((units * waves, width), -1)
    fill = np.zeros(units * waves, int)
    for i in ids:
        members[grp[i], fill[grp[i]]] = i
        fill[grp[i]] += 1
    m = sqdist(x, x[0]).astype(f32)
    out = [0]
    tv, ti = wave_tops(m, members, keep)       # the reports, exact at first
    pending = False                            # picks made since those reports
    rounds = empty = 0
    while len(out) < M:
        rounds += 1
        cid = ti[:, :keep].reshape(units, waves * keep)
        cval = np.where(cid >= 0, m[np.maximum(cid, 0)], f32(-1))      # candidates: exact values
        old_bound = tv[:, keep].reshape(units, waves).max(1)           # bounds: as reported
        order = np.lexsort((cid, -cval), axis=1)
        cs, ci = np.take_along_axis(cval, order, 1), np.take_along_axis(cid, order, 1)
        next_best = cs[:, keep] if cs.shape[1] > keep else np.full(units, f32(-1))
        bound = np.maximum(next_best, old_bound)
        T = bound.max()
        cv, cc = cs[:, :keep].ravel(), ci[:, :keep].ravel()
        live = np.flatnonzero(cv > T)
        if len(live) > max_live:
            live = live[np.lexsort((cc[live], -cv[live]))][:max_live]
            T = max(T, np.sort(cv)[-max_live - 1])
            live = live[cv[live] > T]
        picks = []
        if len(live):
            o = live[np.lexsort((cc[live], -cv[live]))]
            cur = cv[o].copy()
            for k, c in enumerate(o):           # greedy on the candidates, each pick above T
                j = int(np.lexsort((cc[o], -cur))[0])
                if cur[j] <= T or len(out) + len(picks) >= M:
                    break
                picks.append(int(cc[o][j]))
                cur = np.minimum(cur, sqdist(x[cc[o]], x[cc[o][j]]).astype(f32))
                cur[j] = f32(-1)
        elif not pending:
            # exact reports: the best candidate is the best point of all
            j = int(np.lexsort((cc, -cv))[0])
            picks.append(int(cc[j]))
        else:
            empty += 1
        # the workers report the state BEFORE these picks (that is what the next round gets) ...
        if picks or pending:
            tv, ti = wave_tops(m, members, keep)
        # ... and apply them
        for p in picks:
            m = np.minimum(m, sqdist(x, x[p]).astype(f32))
        out += picks
        pending = bool(picks)
    return np.array(out[:M], dtype=np.int32), rounds, empty


@pytest.mark.parametrize("config,n,M,units,waves", [
    (4, 6000, 1500, 16, 7),
    (5, 5000, 800, 8, 7),
    (1, 1024, 512, 4, 3),
    (3, 4096, 1024, 32, 1),
])
def test_overlapped_rounds_pick_what_eq1_picks(oracle, config, n, M, units, waves):
    x = inputs.make_config(config, B=1, N=n)[0]
    got, rounds, empty = overlapped_fps(x, M, units, waves)
    want = oracle.fps_exact(x, M, 0)
    assert np.array_equal(got, want)
    assert rounds < M - 1            # rounds of many picks, not one pick each
    assert empty <= (rounds + 1) // 2  # a round without a pick is followed by one with exact reports, which picks


def test_overlapped_rounds_with_ties(oracle):
    """A lattice: equal distances everywhere, so the tie rule (lowest index) decides often."""
    g = np.arange(12, dtype=f32)
    x = np.stack(np.meshgrid(g, g, g, indexing="ij"), -1).reshape(-1, 3)
    x = x[np.random.default_rng(3).permutation(len(x))].copy()
    got, _, _ = overlapped_fps(x, 400, 8, 4)
    assert np.array_equal(got, oracle.fps_exact(x, 400, 0))
