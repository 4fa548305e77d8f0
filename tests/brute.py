"""Brute-force graph routines used to pin the CPU oracle (numpy only, no oracle code).

Distances come from Floyd-Warshall over the explicit adjacency matrix of the grid graph; regions
from the reachability relation (a component is counted at its lowest-index cell).  Neither a
queue nor a flood fill appears here, so agreement with the oracle is agreement of two different
algorithms on the same textbook objects.
"""
import numpy as np

WALL = 1
INF = 10**6


def passable(tiles):
    t = np.asarray(tiles)
    return (t >= 0) & (t != WALL)


def all_pairs(tiles):
    """[h*w, h*w] shortest-path edge counts between passable cells (INF when none)."""
    p = passable(tiles)
    h, w = p.shape
    n = h * w
    d = np.full((n, n), INF, np.int64)
    for y in range(h):
        for x in range(w):
            if not p[y, x]:
                continue
            i = y * w + x
            d[i, i] = 0
            if x + 1 < w and p[y, x + 1]:
                d[i, i + 1] = d[i + 1, i] = 1
            if y + 1 < h and p[y + 1, x]:
                d[i, i + w] = d[i + w, i] = 1
    for k in range(n):
        d = np.minimum(d, d[:, k:k + 1] + d[k:k + 1, :])
    return d


def regions(tiles, d=None):
    d = all_pairs(tiles) if d is None else d
    n = d.shape[0]
    count = 0
    for i in range(n):
        if d[i, i] != 0:
            continue
        if not np.any(d[i, :i] < INF):
            count += 1
    return count


def two_pass(tiles, d=None):
    """(value, ecc of the start tile, true diameter of the start tile's component)."""
    d = all_pairs(tiles) if d is None else d
    n = d.shape[0]
    cells = [i for i in range(n) if d[i, i] == 0]
    if not cells:
        return 0, 0, 0
    x = cells[0]
    row = np.where(d[x] < INF, d[x], -1)
    far = row.max()
    y = int(np.argmax(row == far))          # lowest index among the farthest
    rowy = np.where(d[y] < INF, d[y], -1)
    comp = [i for i in cells if d[x, i] < INF]
    sub = d[np.ix_(comp, comp)]
    return int(rowy.max()), int(far), int(sub.max())


def nearest(tiles, src_tile, dst_tile, d=None):
    t = np.asarray(tiles).ravel()
    d = all_pairs(tiles) if d is None else d
    s = np.flatnonzero(t == src_tile)
    e = np.flatnonzero(t == dst_tile)
    if len(s) == 0 or len(e) == 0:
        return 0
    m = d[np.ix_(s, e)].min()
    return 0 if m >= INF else int(m)


def dungeon_path(tiles, d=None, player=2, key=3, door=4):
    t = np.asarray(tiles).ravel()
    d = all_pairs(tiles) if d is None else d
    P, Kk, D = (np.flatnonzero(t == v) for v in (player, key, door))
    if len(P) == 0 or len(Kk) == 0 or len(D) == 0:
        return 0
    dk = d[np.ix_(P, Kk)].min(axis=0)       # distance of each key from the nearest player
    d1 = dk.min()
    if d1 >= INF:
        return 0
    k1 = Kk[dk == d1]
    d2 = d[np.ix_(k1, D)].min()
    if d2 >= INF:
        return 0
    return int(d1 + d2)


# ---- the same, vectorised over a stack of equally sized levels ----

def all_pairs_batch(tiles):
    p = passable(tiles)
    N, h, w = p.shape
    n = h * w
    pf = p.reshape(N, n)
    d = np.full((N, n, n), INF, np.int32)
    idx = np.arange(n)
    d[:, idx, idx] = np.where(pf, 0, INF)
    for y in range(h):
        for x in range(w):
            i = y * w + x
            if x + 1 < w:
                e = np.where(pf[:, i] & pf[:, i + 1], 1, INF)
                d[:, i, i + 1] = e
                d[:, i + 1, i] = e
            if y + 1 < h:
                e = np.where(pf[:, i] & pf[:, i + w], 1, INF)
                d[:, i, i + w] = e
                d[:, i + w, i] = e
    for k in range(n):
        d = np.minimum(d, d[:, :, k:k + 1] + d[:, k:k + 1, :])
    return d


def regions_batch(d):
    N, n, _ = d.shape
    reach = d < INF
    count = np.zeros(N, np.int64)
    for i in range(n):
        lower = reach[:, i, :i].any(axis=1) if i else np.zeros(N, bool)
        count += reach[:, i, i] & ~lower
    return count


def two_pass_batch(d):
    """value, ecc(x), diameter of x's component for each level of the stack."""
    N, n, _ = d.shape
    reach = d < INF
    has = reach[:, np.arange(n), np.arange(n)]
    any_cell = has.any(axis=1)
    x = np.argmax(has, axis=1)
    ar = np.arange(N)
    row = np.where(reach[ar, x], d[ar, x], -1)
    far = row.max(axis=1)
    y = np.argmax(row == far[:, None], axis=1)
    rowy = np.where(reach[ar, y], d[ar, y], -1)
    val = rowy.max(axis=1)
    comp = reach[ar, x]                                # cells of x's component
    dd = np.where(comp[:, :, None] & comp[:, None, :] & reach, d, -1)
    diam = dd.reshape(N, -1).max(axis=1)
    z = np.zeros(N, np.int64)
    return (np.where(any_cell, val, z), np.where(any_cell, far, z), np.where(any_cell, diam, z))
