"""ctypes binding of the CPU oracle -- TEST INFRASTRUCTURE, NOT THE PRODUCT.

Only tests, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of ``bench.py`` may import
this package.  It wraps ``pcgrl_oracle.c`` (plain C, one cell at a time) and holds no arithmetic
of its own: every function below only marshals numpy arrays.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "pcgrl_oracle.c")
_HDR = os.path.join(_HERE, "pcgrl_oracle.h")
_LIB = os.path.join(_HERE, "libpcgrl_oracle.so")

BINARY, MAZE, DUNGEON = 0, 1, 2
PAD_BORDER, PAD_WALL = 0, 1
POS_SCAN, POS_RANDOM = 0, 1
MAX_METRICS, MAX_TILES = 16, 8


class OrcConfig(C.Structure):
    _fields_ = [
        ("problem", C.c_int32), ("batch", C.c_int32),
        ("max_h", C.c_int32), ("max_w", C.c_int32),
        ("min_h", C.c_int32), ("min_w", C.c_int32),
        ("obs_w", C.c_int32), ("pad_mode", C.c_int32), ("pos_mode", C.c_int32),
        ("n_frozen", C.c_int32), ("max_steps", C.c_int32), ("max_changes", C.c_int32),
        ("autoreset", C.c_int32),
        ("init_cdf", C.c_uint32 * MAX_TILES),
        ("weights", C.c_float * MAX_METRICS),
        ("target_lo", C.c_int32 * MAX_METRICS),
        ("target_hi", C.c_int32 * MAX_METRICS),
        ("pinpoint_tile", C.c_int32 * 8),
        ("ctrl_mask", C.c_uint32),
        ("ctrl_lo", C.c_int32 * MAX_METRICS),
        ("ctrl_hi", C.c_int32 * MAX_METRICS),
        ("obs_frozen_channel", C.c_int32),
    ]


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no contraction of float multiply-add, no vector tricks)."""
    stale = (not os.path.exists(_LIB)
             or os.path.getmtime(_LIB) < max(os.path.getmtime(_SRC), os.path.getmtime(_HDR)))
    if force or stale:
        subprocess.check_call(["gcc", "-std=c11", "-O2", "-ffp-contract=off", "-fPIC", "-shared",
                               "-Wall", "-Wextra", "-o", _LIB, _SRC])
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(build())
        p = C.c_void_p
        L.orc_create.restype = p
        L.orc_create.argtypes = [C.POINTER(OrcConfig)]
        L.orc_destroy.argtypes = [p]
        L.orc_reset.argtypes = [p, C.c_uint64, p]
        L.orc_step.argtypes = [p, p, p, p, p]
        L.orc_step_range.argtypes = [p, C.c_int, C.c_int, p, p, p, p]
        L.orc_metrics.argtypes = [p, p]
        L.orc_observe.argtypes = [p, p]
        L.orc_exact_diameters.argtypes = [p, p]
        L.orc_exact_diameter.argtypes = [p, C.c_int, C.c_int, C.c_int]
        L.orc_get_state.argtypes = [p, p, p, p, p, p]
        L.orc_set_state.argtypes = [p, p, p, p, p]
        L.orc_set_targets.argtypes = [p, p]
        L.orc_get_targets.argtypes = [p, p]
        L.orc_mix64.restype = C.c_uint64
        L.orc_mix64.argtypes = [C.c_uint64]
        L.orc_env_key.restype = C.c_uint64
        L.orc_env_key.argtypes = [C.c_uint64] * 3
        L.orc_draw.restype = C.c_uint64
        L.orc_draw.argtypes = [C.c_uint64, C.c_uint32, C.c_uint32]
        L.orc_below.argtypes = [C.c_uint32, C.c_int]
        L.orc_regions.argtypes = [p, C.c_int, C.c_int, C.c_int]
        L.orc_bfs.argtypes = [p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, p]
        L.orc_diameter_two_pass.argtypes = [p, C.c_int, C.c_int, C.c_int]
        L.orc_path_nearest.argtypes = [p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int]
        L.orc_path_dungeon.argtypes = [p, C.c_int, C.c_int, C.c_int]
        L.orc_level_metrics.argtypes = [C.c_int, p, C.c_int, C.c_int, C.c_int, p]
        L.orc_loss.argtypes = [C.c_int] * 3
        L.orc_num_tiles.argtypes = [C.c_int]
        L.orc_num_metrics.argtypes = [C.c_int]
        L.orc_num_channels.argtypes = [C.POINTER(OrcConfig)]
        _lib = L
    return _lib


def _ptr(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def make_config(d: dict) -> OrcConfig:
    """Fill the oracle's own config struct from a plain dict of fields."""
    c = OrcConfig()
    known = {f[0] for f in OrcConfig._fields_}
    for k, v in d.items():
        if k not in known:      # knobs of other implementations (e.g. how regions are counted)
            continue
        if k in ("init_cdf", "weights", "target_lo", "target_hi", "pinpoint_tile", "ctrl_lo", "ctrl_hi"):
            arr = getattr(c, k)
            for i, x in enumerate(v):
                arr[i] = x
        else:
            setattr(c, k, int(v))
    return c


class Oracle:
    """One batch of oracle environments; all arrays are host numpy arrays."""

    def __init__(self, cfg: dict):
        self.cfg = make_config(cfg)
        self.L = lib()
        self.h = self.L.orc_create(C.byref(self.cfg))
        if not self.h:
            raise ValueError("oracle rejected the configuration")
        self.B = self.cfg.batch
        self.K = self.L.orc_num_tiles(self.cfg.problem)
        self.M = self.L.orc_num_metrics(self.cfg.problem)
        self.Cn = self.L.orc_num_channels(C.byref(self.cfg))
        self.ow = self.cfg.obs_w
        self.Hm, self.Wm = self.cfg.max_h, self.cfg.max_w

    def __del__(self):
        if getattr(self, "h", None):
            self.L.orc_destroy(self.h)
            self.h = None

    def new_obs(self):
        return np.zeros((self.B, self.Cn, self.ow, self.ow), np.uint8)

    def reset(self, seed: int, want_obs: bool = True):
        obs = self.new_obs() if want_obs else None
        self.L.orc_reset(self.h, C.c_uint64(seed), _ptr(obs))
        return obs

    def step(self, actions, want_obs: bool = True):
        actions = np.ascontiguousarray(actions, np.int32)
        assert actions.shape == (self.B,)
        obs = self.new_obs() if want_obs else None
        rew = np.zeros(self.B, np.float32)
        done = np.zeros(self.B, np.uint8)
        self.L.orc_step(self.h, _ptr(actions), _ptr(obs), _ptr(rew), _ptr(done))
        return obs, rew, done

    def step_range(self, lo, hi, actions, obs, rew, done):
        """Step envs [lo, hi) into caller-owned output arrays (for threaded timing)."""
        self.L.orc_step_range(self.h, lo, hi, _ptr(actions), _ptr(obs), _ptr(rew), _ptr(done))

    def metrics(self):
        out = np.zeros((self.B, self.M), np.int32)
        self.L.orc_metrics(self.h, _ptr(out))
        return out

    def exact_diameters(self):
        out = np.zeros(self.B, np.int32)
        self.L.orc_exact_diameters(self.h, _ptr(out))
        return out

    def observe(self):
        obs = self.new_obs()
        self.L.orc_observe(self.h, _ptr(obs))
        return obs

    def get_state(self):
        tiles = np.zeros((self.B, self.Hm, self.Wm), np.int8)
        frozen = np.zeros((self.B, self.Hm, self.Wm), np.uint8)
        hw = np.zeros((self.B, 2), np.int16)
        pos = np.zeros((self.B, 2), np.int16)
        ctr = np.zeros((self.B, 3), np.int32)
        self.L.orc_get_state(self.h, _ptr(tiles), _ptr(frozen), _ptr(hw), _ptr(pos), _ptr(ctr))
        return dict(tiles=tiles, frozen=frozen, hw=hw, pos=pos, counters=ctr)

    def set_state(self, tiles, frozen, hw, pos):
        tiles = np.ascontiguousarray(tiles, np.int8)
        frozen = None if frozen is None else np.ascontiguousarray(frozen, np.uint8)
        hw = np.ascontiguousarray(hw, np.int16)
        pos = np.ascontiguousarray(pos, np.int16)
        assert tiles.shape == (self.B, self.Hm, self.Wm)
        assert hw.shape == (self.B, 2) and pos.shape == (self.B, 2)
        self.L.orc_set_state(self.h, _ptr(tiles), _ptr(frozen), _ptr(hw), _ptr(pos))

    def get_targets(self):
        out = np.zeros((self.B, self.M, 2), np.int32)
        self.L.orc_get_targets(self.h, _ptr(out))
        return out

    def set_targets(self, targets):
        targets = np.ascontiguousarray(targets, np.int32)
        assert targets.shape == (self.B, self.M, 2)
        self.L.orc_set_targets(self.h, _ptr(targets))


# ---- single-level building blocks (tiles: int8 [h, w]) ----

def _lvl(tiles):
    t = np.ascontiguousarray(tiles, np.int8)
    assert t.ndim == 2
    return t, t.shape[0], t.shape[1]


def regions(tiles) -> int:
    t, h, w = _lvl(tiles)
    return lib().orc_regions(_ptr(t), h, w, w)


def bfs(tiles, src_tile=-1, src_index=0):
    t, h, w = _lvl(tiles)
    dist = np.zeros((h, w), np.int32)
    lib().orc_bfs(_ptr(t), h, w, w, src_tile, src_index, _ptr(dist))
    return dist


def diameter_two_pass(tiles) -> int:
    t, h, w = _lvl(tiles)
    return lib().orc_diameter_two_pass(_ptr(t), h, w, w)


def exact_diameter(tiles) -> int:
    t, h, w = _lvl(tiles)
    return lib().orc_exact_diameter(_ptr(t), h, w, w)


def path_nearest(tiles, src_tile, dst_tile) -> int:
    t, h, w = _lvl(tiles)
    return lib().orc_path_nearest(_ptr(t), h, w, w, src_tile, dst_tile)


def path_dungeon(tiles) -> int:
    t, h, w = _lvl(tiles)
    return lib().orc_path_dungeon(_ptr(t), h, w, w)


def level_metrics(problem, tiles):
    t, h, w = _lvl(tiles)
    m = np.zeros(lib().orc_num_metrics(problem), np.int32)
    lib().orc_level_metrics(problem, _ptr(t), h, w, w, _ptr(m))
    return m


def loss(v, lo, hi) -> int:
    return lib().orc_loss(int(v), int(lo), int(hi))


def mix64(z) -> int:
    return lib().orc_mix64(C.c_uint64(z & (2**64 - 1)))


def env_key(seed, env, episode) -> int:
    return lib().orc_env_key(C.c_uint64(seed), C.c_uint64(env), C.c_uint64(episode))


def draw(key, stream, counter) -> int:
    return lib().orc_draw(C.c_uint64(key), C.c_uint32(stream), C.c_uint32(counter))


def below(r, n) -> int:
    return lib().orc_below(C.c_uint32(r), int(n))
