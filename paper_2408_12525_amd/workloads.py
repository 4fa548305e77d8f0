"""Seeded synthetic workloads: configuration tables and action generators.

This module holds data only (field values, probabilities, weights, target ranges) and draws the
agents' random actions; none of the environment's arithmetic lives here.  Both the GPU library's
binding and the tests' CPU oracle are fed from it, so that they see identical inputs.

The paper's environments are procedurally generated (Methods / Task: weighted random initial
map; Results / Speed comparison: actions from a random agent), so seeded synthetic levels and
uniform random actions *are* the workload shape; no dataset stands behind them.
"""
from __future__ import annotations

import numpy as np

BINARY, MAZE, DUNGEON = 0, 1, 2
PAD_BORDER, PAD_WALL = 0, 1
POS_SCAN, POS_RANDOM = 0, 1
REGIONS_INCREMENTAL, REGIONS_RECOUNT = 0, 1

NUM_TILES = {BINARY: 2, MAZE: 4, DUNGEON: 7}
# a target no path length can reach: "maximise" is "get as close to BIG as possible"
BIG = 64 * 64


def num_metrics(problem: int) -> int:
    return (3 if problem == DUNGEON else 2) + NUM_TILES[problem]


def metric_names(problem: int):
    if problem == BINARY:
        return ["regions", "diameter", "n_empty", "n_wall"]
    if problem == MAZE:
        return ["regions", "path", "n_empty", "n_wall", "n_player", "n_door"]
    return ["regions", "path", "nearest_enemy", "n_empty", "n_wall", "n_player", "n_key",
            "n_door", "n_enemy", "n_chest"]


def default_reward_table(problem: int):
    """(weights, target_lo, target_hi) per metric.

    Targets follow the problem statements (one region; path as long as possible; exactly one
    player / key / door; two to five enemies; nearest enemy at least four tiles away).  The
    weights are this build's own small integers: the paper takes them from code bases it cites
    but does not print, so they are inputs here, never constants of the library.
    """
    if problem == BINARY:
        w = [5, 2, 0, 0]
        lo = [1, BIG, 0, 0]
        hi = [1, BIG, BIG, BIG]
    elif problem == MAZE:
        w = [5, 2, 0, 0, 3, 3]
        lo = [1, BIG, 0, 0, 1, 1]
        hi = [1, BIG, BIG, BIG, 1, 1]
    else:
        #    reg path  ne  emp wall ply key door enemy chest
        w = [5, 2, 2, 0, 0, 3, 3, 3, 3, 0]
        lo = [1, BIG, 4, 0, 0, 1, 1, 1, 2, 0]
        hi = [1, BIG, BIG, BIG, BIG, 1, 1, 1, 5, BIG]
    return [float(x) for x in w], lo, hi


def cdf_from_probs(probs):
    """Cumulative 32-bit thresholds of a tile distribution (last one saturates)."""
    acc, out = 0.0, []
    for p in probs:
        acc += float(p)
        out.append(min(2**32 - 1, int(round(acc * 2**32))))
    out[-1] = 2**32 - 1
    return out + [0] * (8 - len(out))


def make_config(problem, batch, size, obs_w, *, min_size=None, pad_mode=PAD_BORDER,
                pos_mode=POS_RANDOM, n_frozen=0, max_steps=1000, max_changes=0, autoreset=1,
                probs=None, weights=None, target_lo=None, target_hi=None, max_w=None,
                min_w=None, regions_mode=REGIONS_INCREMENTAL, levels_per_wave=0,
                obs_store_mode=0, split_step=0, obs_format=0, pinpoint_tile=None, ctrl=None,
                obs_frozen_channel=0, split_obs_levels=0, obs_pitch=0, rollout_turns=0):
    """ctrl: {metric index: (lo, hi)} -- targets drawn per episode; pinpoint_tile: tile of each
    pinpoint (-1 keeps the drawn one)."""
    w, lo, hi = default_reward_table(problem)
    mh = size
    mw = size if max_w is None else max_w
    nh = mh if min_size is None else min_size
    nw = (mw if min_size is None else min_size) if min_w is None else min_w
    K = NUM_TILES[problem]
    if probs is None:                       # probs="empty" starts from an all-empty map
        probs = [1.0 / K] * K
    pad16 = lambda v, z: list(v) + [z] * (16 - len(v))
    ctrl = ctrl or {}
    pin = list(pinpoint_tile or []) + [-1] * 8
    return dict(
        problem=problem, batch=batch, max_h=mh, max_w=mw, min_h=nh, min_w=nw, obs_w=obs_w,
        pad_mode=pad_mode, pos_mode=pos_mode, n_frozen=n_frozen, max_steps=max_steps,
        max_changes=max_changes, autoreset=autoreset,
        init_cdf=[0] * 8 if isinstance(probs, str) else cdf_from_probs(probs),
        weights=pad16(weights if weights is not None else w, 0.0)[:16],
        target_lo=pad16(target_lo if target_lo is not None else lo, 0)[:16],
        target_hi=pad16(target_hi if target_hi is not None else hi, 0)[:16],
        regions_mode=regions_mode, levels_per_wave=levels_per_wave,
        obs_store_mode=obs_store_mode, split_step=split_step, obs_format=obs_format,
        pinpoint_tile=pin[:8],
        ctrl_mask=sum(1 << i for i in ctrl),
        ctrl_lo=[ctrl.get(i, (0, 0))[0] for i in range(16)],
        ctrl_hi=[ctrl.get(i, (0, 0))[1] for i in range(16)],
        obs_frozen_channel=obs_frozen_channel, split_obs_levels=split_obs_levels,
        obs_pitch=obs_pitch, rollout_turns=rollout_turns,
    )


# The five workload shapes this build is measured and checked on.
def workload(name: str, batch: int | None = None, **over):
    if name == "binary16":      # 16x16 binary, Bernoulli(0.5) start, full-map view, wall padding
        c = make_config(BINARY, 64, 16, 31, pad_mode=PAD_WALL, max_steps=1000, probs=[.5, .5])
    elif name == "maze16":      # 16x16 maze
        c = make_config(MAZE, 4096, 16, 31, max_steps=10000, probs=[.45, .45, .05, .05])
    elif name.startswith("binary32_rand"):   # randomized shape in a 32x32 buffer, 3 pinpoints
        ow = int(name.split("_ow")[1]) if "_ow" in name else 15
        c = make_config(BINARY, 16384, 32, ow, min_size=8, n_frozen=3, max_steps=1000,
                        probs=[.5, .5])
    elif name == "maze64":      # out-of-distribution 64x64 maze
        c = make_config(MAZE, 8192, 64, 31, max_steps=1000, probs=[.45, .45, .05, .05])
    elif name == "dungeon32":   # 7-tile dungeon
        c = make_config(DUNGEON, 16384, 32, 15, max_steps=1000,
                        probs=[.40, .40, .04, .04, .04, .04, .04])
    elif name == "maze16_pinpoint":   # empty start, frozen player and door, random shape 3..16
        c = make_config(MAZE, 4096, 16, 8, min_size=3, probs="empty", n_frozen=2, pinpoint_tile=[2, 3],
                        max_steps=1000)
    elif name == "dungeon16_ctrl":    # dungeon with a controllable path length and nearest enemy
        c = make_config(DUNGEON, 4096, 16, 31, max_steps=1000, n_frozen=3, pinpoint_tile=[2, 3, 4],
                        probs=[.40, .40, .04, .04, .04, .04, .04], ctrl={1: (10, 60), 2: (2, 9)})
    else:
        raise KeyError(name)
    if batch is not None:
        c["batch"] = batch
    c.update(over)
    return c


WORKLOADS = ["binary16", "maze16", "binary32_rand_ow3", "binary32_rand_ow15",
             "binary32_rand_ow63", "maze64", "dungeon32"]


def random_actions(cfg: dict, seed: int, steps: int, bad_fraction: float = 0.0):
    """int32 [steps, batch] uniform over the problem's tiles (a random agent).

    ``bad_fraction`` > 0 replaces that share of the actions by out-of-range values, which the
    environment must treat as no-ops.
    """
    K = NUM_TILES[cfg["problem"]]
    rng = np.random.Generator(np.random.PCG64(seed))
    a = rng.integers(0, K, size=(steps, cfg["batch"]), dtype=np.int32)
    if bad_fraction > 0:
        bad = rng.random((steps, cfg["batch"])) < bad_fraction
        junk = rng.choice(np.array([-1, K, K + 5, 127, -2**31], np.int64), size=a.shape)
        a = np.where(bad, junk, a).astype(np.int32)
    return a


def obs_bytes(cfg: dict) -> int:
    C = (NUM_TILES[cfg["problem"]] + (1 if cfg["pad_mode"] == PAD_BORDER else 0)
         + (1 if cfg.get("obs_frozen_channel", 0) else 0))
    cells = C * cfg["obs_w"] * cfg["obs_w"]
    return (cells + 7) // 8 if cfg.get("obs_format", 0) else cells
