"""Pins of the CPU oracle's building blocks against things that are not the oracle:
published generator outputs, closed forms on hand-built levels, and brute force on tiny maps.
CPU only."""
import numpy as np
import pytest

import brute
import levels
import oracle
from paper_2408_12525_amd import workloads as wl


# ---------------------------------------------------------------- generator

def test_mix64_reproduces_published_splitmix64_sequence():
    # First five outputs of splitmix64 seeded with 1234567, as printed with the generator's
    # public-domain reference code: the state advances by the golden-ratio constant, the output
    # is the mixing function of the new state.
    want = [6457827717110365317, 3203168211198807973, 9817491932198370423,
            4593380528125082431, 16408922859458223821]
    s, got = 1234567, []
    for _ in range(5):
        s = (s + 0x9E3779B97F4A7C15) % 2**64
        got.append(oracle.mix64(s))
    assert got == want


def test_keys_and_draws_do_not_collide():
    keys = {oracle.env_key(7, e, ep) for e in range(64) for ep in range(8)}
    assert len(keys) == 64 * 8
    k = oracle.env_key(7, 3, 0)
    draws = {oracle.draw(k, s, c) for s in range(4) for c in range(4096)}
    assert len(draws) == 4 * 4096
    assert oracle.env_key(7, 3, 0) != oracle.env_key(8, 3, 0)


# ----------------------------------------------------- hand-built fixtures

@pytest.mark.parametrize("name", levels.all_fixtures())
def test_hand_built_level(name):
    problem, tiles, expect = levels.load(name)
    pid = levels.PROBLEM_ID[problem]
    m = oracle.level_metrics(pid, tiles)
    got = dict(zip(wl.metric_names(pid), (int(v) for v in m)))
    if "exact_diameter" in expect:
        assert oracle.exact_diameter(tiles) == expect.pop("exact_diameter"), name
    for k, v in expect.items():
        assert got[k] == v, (name, k, got)
    # the same level embedded in a larger buffer (row pitch != width) must read the same
    big = np.full((tiles.shape[0] + 2, tiles.shape[1] + 3), -1, np.int8)
    big[:tiles.shape[0], :tiles.shape[1]] = tiles
    m2 = np.zeros_like(m)
    oracle.lib().orc_level_metrics(pid, big.ctypes.data, tiles.shape[0], tiles.shape[1],
                                   big.shape[1], m2.ctypes.data)
    assert (m2 == m).all()


# ------------------------------------------------ exhaustive / brute force

def test_every_4x4_binary_map_regions_and_two_pass():
    N = 1 << 16
    maps = ((np.arange(N)[:, None] >> np.arange(16)) & 1).astype(np.int8).reshape(N, 4, 4)
    d = brute.all_pairs_batch(maps)
    reg = brute.regions_batch(d)
    val, eccx, diam = brute.two_pass_batch(d)
    assert (eccx <= val).all() and (val <= diam).all()     # ecc(x) <= ecc(y) <= diameter
    for i in range(N):
        assert oracle.regions(maps[i]) == reg[i], i
        assert oracle.diameter_two_pass(maps[i]) == val[i], i


def _random_level(rng, K, h, w, p_wall):
    probs = np.full(K, (1 - p_wall) / (K - 1))
    probs[1] = p_wall
    return rng.choice(K, size=(h, w), p=probs).astype(np.int8)


@pytest.mark.parametrize("seed", range(4))
def test_random_small_maps_all_metrics_vs_brute_force(seed):
    rng = np.random.default_rng(seed)
    for _ in range(150):
        h, w = rng.integers(1, 7, size=2)
        p_wall = rng.choice([0.1, 0.3, 0.5, 0.7])
        # binary
        t = _random_level(rng, 2, h, w, p_wall)
        d = brute.all_pairs(t)
        m = oracle.level_metrics(wl.BINARY, t)
        assert m[0] == brute.regions(t, d)
        assert m[1] == brute.two_pass(t, d)[0]
        assert m[2] == (t == 0).sum() and m[3] == (t == 1).sum()
        # maze
        t = _random_level(rng, 4, h, w, p_wall)
        d = brute.all_pairs(t)
        m = oracle.level_metrics(wl.MAZE, t)
        assert m[0] == brute.regions(t, d)
        assert m[1] == brute.nearest(t, 2, 3, d)
        assert [m[2 + k] for k in range(4)] == [(t == k).sum() for k in range(4)]
        # dungeon
        t = _random_level(rng, 7, h, w, p_wall)
        d = brute.all_pairs(t)
        m = oracle.level_metrics(wl.DUNGEON, t)
        assert m[0] == brute.regions(t, d)
        assert m[1] == brute.dungeon_path(t, d)
        assert m[2] == brute.nearest(t, 2, 5, d)
        assert [m[3 + k] for k in range(7)] == [(t == k).sum() for k in range(7)]


def test_bfs_distance_field_vs_all_pairs():
    rng = np.random.default_rng(11)
    for _ in range(60):
        h, w = rng.integers(2, 8, size=2)
        t = _random_level(rng, 2, h, w, 0.35)
        d = brute.all_pairs(t)
        free = np.flatnonzero(brute.passable(t).ravel())
        if len(free) == 0:
            continue
        s = int(rng.choice(free))
        got = oracle.bfs(t, -1, s).ravel()
        want = np.where(d[s] < brute.INF, d[s], -1)
        assert (got == want).all()


def test_single_instance_dungeon_is_sum_of_two_distances():
    # with one player, key and door the reading must reduce to dist(p,k) + dist(k,d)
    rng = np.random.default_rng(5)
    done = 0
    while done < 80:
        h, w = rng.integers(3, 7, size=2)
        t = _random_level(rng, 2, h, w, 0.25)
        free = np.flatnonzero(t.ravel() == 0)
        if len(free) < 3:
            continue
        p, k, dd = rng.choice(free, 3, replace=False)
        t.ravel()[p], t.ravel()[k], t.ravel()[dd] = 2, 3, 4
        d = brute.all_pairs(t)
        want = 0 if d[p, k] >= brute.INF or d[k, dd] >= brute.INF else d[p, k] + d[k, dd]
        assert oracle.path_dungeon(t) == want
        done += 1


def test_exact_diameter_vs_all_pairs():
    rng = np.random.default_rng(21)
    for _ in range(120):
        h, w = rng.integers(1, 8, size=2)
        t = _random_level(rng, 4, h, w, rng.choice([0.1, 0.3, 0.5]))
        d = brute.all_pairs(t)
        fin = d[d < brute.INF]
        want = int(fin.max()) if fin.size else 0
        got = oracle.exact_diameter(t)
        assert got == want
        if (t != 1).any():
            m = oracle.level_metrics(wl.BINARY, (t == 1).astype(np.int8))
            assert m[1] <= got                    # the two-sweep value never exceeds the diameter


def test_loss_is_distance_to_range():
    for v in range(-3, 12):
        for lo in range(0, 6):
            for hi in range(lo, 8):
                want = 0 if lo <= v <= hi else min(abs(v - lo), abs(v - hi))
                assert oracle.loss(v, lo, hi) == want
