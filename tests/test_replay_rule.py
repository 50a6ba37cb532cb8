"""The rule by which a round's picks are settled from pairwise bit masks
(paper_2604_17720_amd/csrc/fps_exchange.h: team_matrix and the settle step of
replay_round), written out in NumPy and checked against the greedy rule of
Eq. 1 run pick after pick on the same candidates.

This is a statement about the rule, not about the kernels (those are compared
with the oracle element by element in the GPU tests): for candidates with
values o above a threshold T, where every point that is not a candidate is at
or below T, the rule must return a prefix of what the greedy loop returns."""
import numpy as np


def greedy(pts, o, idx, T, cap):
    """Eq. 1 on the candidates alone: largest current value, lowest index among
    equals; stops when the best value is not above T (an unreported point might
    be the maximum then) or after cap picks."""
    n = len(o)
    cur = o.copy()
    picked = np.zeros(n, bool)
    out = []
    while len(out) < cap:
        best = max((i for i in range(n) if not picked[i]), key=lambda i: (cur[i], -idx[i]), default=None)
        if best is None or cur[best] <= T:
            break
        out.append(best)
        picked[best] = True
        cur = np.minimum(cur, ((pts - pts[best]) ** 2).sum(1))
    return out


def settle(pts, o, idx, T, cap):
    """The masks and the passes over them, as the kernels do it."""
    n = len(o)
    d = ((pts[:, None, :] - pts[None, :, :]) ** 2).sum(2)
    key = [(o[i], -idx[i]) for i in range(n)]
    before = np.array([[key[a] > key[b] for b in range(n)] for a in range(n)])    # a before b
    out_of_round = (d <= T) & before
    lowers = (d < o[None, :]) & before
    pick = np.ones(n, bool)
    for _ in range(n + 1):          # b is a pick iff no pick before it lowers it
        nxt = ~((lowers & pick[:, None]).any(0))
        if (nxt == pick).all():
            break
        pick = nxt
    gone = ~pick & (out_of_round & pick[:, None]).any(0)
    wounded = ~pick & ~gone        # lowered, still above T: its new value ends the round
    vstar = 0.0
    for b in np.nonzero(wounded)[0]:
        vstar = max(vstar, d[np.nonzero(lowers[:, b] & pick)[0], b].min())
    final = pick & (o > vstar)
    order = (before & final[:, None]).sum(0)
    return sorted((b for b in range(n) if final[b] and order[b] < cap), key=lambda b: order[b])


def test_mask_rule_returns_a_prefix_of_the_greedy_sequence():
    rng = np.random.default_rng(7)
    total = 0
    for _ in range(1500):
        n = int(rng.integers(1, 80))
        pts = rng.integers(0, 14, size=(n, 3)).astype(float)      # small lattice: equal distances everywhere
        o = rng.integers(3, 40, size=n).astype(float)             # equal values too
        idx = rng.permutation(1000)[:n]
        T = float(rng.integers(0, 6))
        o = np.maximum(o, T + 1)
        cap = int(rng.integers(1, n + 3))
        want, got = greedy(pts, o, idx, T, cap), settle(pts, o, idx, T, cap)
        assert len(got) >= 1 and want[:len(got)] == got
        total += len(got)
    assert total > 5000
