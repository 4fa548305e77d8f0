"""Thin Python binding of the C ABI in include/pcgrl.h.

Argument marshalling only: tensors are checked (device, dtype, shape, contiguity) and handed over
as raw device pointers together with the current HIP stream.  Every step of the environment runs
in the library's kernels.  There is no fallback: if the compiled library is missing or cannot be
loaded, the first call raises.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

from . import build as _build

MAX_METRICS, MAX_TILES = 16, 8


class PcgrlConfig(C.Structure):
    _fields_ = [
        ("problem", C.c_int32), ("batch", C.c_int32),
        ("max_h", C.c_int32), ("max_w", C.c_int32),
        ("min_h", C.c_int32), ("min_w", C.c_int32),
        ("obs_w", C.c_int32), ("pad_mode", C.c_int32), ("pos_mode", C.c_int32),
        ("n_frozen", C.c_int32), ("max_steps", C.c_int32), ("max_changes", C.c_int32),
        ("autoreset", C.c_int32), ("regions_mode", C.c_int32), ("levels_per_wave", C.c_int32),
        ("obs_store_mode", C.c_int32), ("split_step", C.c_int32),
        ("obs_format", C.c_int32),
        ("init_cdf", C.c_uint32 * MAX_TILES),
        ("weights", C.c_float * MAX_METRICS),
        ("target_lo", C.c_int32 * MAX_METRICS),
        ("target_hi", C.c_int32 * MAX_METRICS),
        ("pinpoint_tile", C.c_int32 * 8),
        ("ctrl_mask", C.c_uint32),
        ("ctrl_lo", C.c_int32 * MAX_METRICS),
        ("ctrl_hi", C.c_int32 * MAX_METRICS),
        ("obs_frozen_channel", C.c_int32),
        ("split_obs_levels", C.c_int32),
        ("obs_pitch", C.c_int32),
        ("rollout_turns", C.c_int32),
    ]


EXPORTS = [
    "pcgrl_config_default", "pcgrl_create", "pcgrl_destroy", "pcgrl_reset", "pcgrl_step", "pcgrl_rollout",
    "pcgrl_metrics", "pcgrl_exact_diameter", "pcgrl_exact_diameter_static", "pcgrl_observe", "pcgrl_get_state", "pcgrl_set_state", "pcgrl_set_targets",
    "pcgrl_get_targets",
    "pcgrl_obs_shape", "pcgrl_obs_bytes", "pcgrl_obs_stride", "pcgrl_num_metrics", "pcgrl_num_tiles", "pcgrl_bad_action_count",
    "pcgrl_selftest", "pcgrl_store_rate", "pcgrl_unpack_obs", "pcgrl_strerror",
]

_lib = None


class PcgrlError(RuntimeError):
    pass


def library_path() -> str:
    return _build.LIB


def load():
    """Loads the in-tree library.  If it has never been built it is compiled first (hipcc); if
    that is impossible the call raises -- there is no other implementation to fall back to."""
    global _lib
    if _lib is not None:
        return _lib
    path = library_path()
    if not os.path.exists(path):
        try:
            _build.build(force=True)
        except Exception as e:  # no hipcc, compile error, read-only tree ...
            raise PcgrlError(f"{path} is missing and could not be built ({e}); "
                             "there is no fallback implementation") from e
    L = C.CDLL(path)
    p, i32, u64 = C.c_void_p, C.c_int32, C.c_uint64
    L.pcgrl_config_default.argtypes = [i32, C.POINTER(PcgrlConfig)]
    L.pcgrl_create.argtypes = [C.POINTER(p), C.POINTER(PcgrlConfig), C.c_int]
    L.pcgrl_destroy.argtypes = [p]
    L.pcgrl_reset.argtypes = [p, u64, p, p]
    L.pcgrl_step.argtypes = [p, p, p, p, p, p]
    L.pcgrl_rollout.argtypes = [p, p, i32, p, i32, p, p, p]
    L.pcgrl_metrics.argtypes = [p, p, p]
    L.pcgrl_observe.argtypes = [p, p, p]
    L.pcgrl_exact_diameter.argtypes = [p, p, p]
    L.pcgrl_exact_diameter_static.argtypes = [p, p, i32, p]
    L.pcgrl_get_state.argtypes = [p, p, p, p, p, p, p]
    L.pcgrl_set_state.argtypes = [p, p, p, p, p, p]
    L.pcgrl_set_targets.argtypes = [p, p, p]
    L.pcgrl_get_targets.argtypes = [p, p, p]
    L.pcgrl_obs_shape.argtypes = [p, C.POINTER(i32 * 4)]
    L.pcgrl_obs_bytes.argtypes = [p]
    L.pcgrl_obs_bytes.restype = C.c_int64
    L.pcgrl_obs_stride.argtypes = [p]
    L.pcgrl_obs_stride.restype = C.c_int64
    L.pcgrl_num_metrics.argtypes = [p]
    L.pcgrl_num_tiles.argtypes = [p]
    L.pcgrl_bad_action_count.argtypes = [p, C.POINTER(u64), p]
    L.pcgrl_selftest.argtypes = [C.c_int, C.POINTER(i32)]
    L.pcgrl_store_rate.argtypes = [p, C.c_int64, i32, i32, i32, p]
    L.pcgrl_unpack_obs.argtypes = [p, p, p, i32, p]
    L.pcgrl_strerror.argtypes = [C.c_int]
    L.pcgrl_strerror.restype = C.c_char_p
    _lib = L
    return L


def _check(rc: int, what: str):
    if rc != 0:
        raise PcgrlError(f"{what} failed: {load().pcgrl_strerror(rc).decode()} ({rc})")


def make_config(d: dict) -> PcgrlConfig:
    c = PcgrlConfig()
    for k, v in d.items():
        if k in ("init_cdf", "weights", "target_lo", "target_hi", "pinpoint_tile", "ctrl_lo", "ctrl_hi"):
            arr = getattr(c, k)
            for i, x in enumerate(v):
                arr[i] = x
        else:
            setattr(c, k, int(v))
    return c


def pcgrl_config_default(problem: int) -> PcgrlConfig:
    c = PcgrlConfig()
    _check(load().pcgrl_config_default(problem, C.byref(c)), "pcgrl_config_default")
    return c


def pcgrl_selftest(device: int = 0) -> int:
    n = C.c_int32(-1)
    _check(load().pcgrl_selftest(device, C.byref(n)), "pcgrl_selftest")
    return n.value


def pcgrl_store_rate(dst, n_regions: int, region_bytes: int, store_mode: int = 1, order: int = 0):
    """One store-only launch over dst (uint8 tensor on the current device); see pcgrl_store_rate."""
    if not (isinstance(dst, torch.Tensor) and dst.is_cuda and dst.dtype == torch.uint8 and dst.is_contiguous()):
        raise PcgrlError("dst must be a contiguous uint8 tensor on the GPU")
    if dst.numel() < n_regions * region_bytes:
        raise PcgrlError("dst is smaller than n_regions * region_bytes")
    _check(load().pcgrl_store_rate(C.c_void_p(dst.data_ptr()), n_regions, region_bytes, store_mode,
                                   int(order), C.c_void_p(_stream_ptr(dst.device))), "pcgrl_store_rate")


def _stream_ptr(device) -> int:
    return torch.cuda.current_stream(device).cuda_stream


class Pcgrl:
    """A batch of GPU-resident environments (one pcgrl_ctx).  Methods carry the C names."""

    def __init__(self, cfg: dict | PcgrlConfig, device: int = 0):
        self.L = load()
        self.cfg = cfg if isinstance(cfg, PcgrlConfig) else make_config(cfg)
        self.device = torch.device("cuda", device)
        self.h = C.c_void_p()
        _check(self.L.pcgrl_create(C.byref(self.h), C.byref(self.cfg), device), "pcgrl_create")
        shp = (C.c_int32 * 4)()
        _check(self.L.pcgrl_obs_shape(self.h, C.byref(shp)), "pcgrl_obs_shape")
        self.obs_shape = tuple(shp)
        self.obs_bytes = int(self.L.pcgrl_obs_bytes(self.h))
        self.obs_stride = int(self.L.pcgrl_obs_stride(self.h))
        self.onehot_shape = tuple(shp)
        if self.cfg.obs_format != 0 or self.obs_stride != self.obs_bytes:
            # bit-packed or pitched: one flat byte row per level
            self.obs_shape = (shp[0], self.obs_stride)
        self.B = self.cfg.batch
        self.M = self.L.pcgrl_num_metrics(self.h)
        self.K = self.L.pcgrl_num_tiles(self.h)
        self.Hm, self.Wm = self.cfg.max_h, self.cfg.max_w

    def close(self):
        if getattr(self, "h", None) is not None and self.h:
            _check(self.L.pcgrl_destroy(self.h), "pcgrl_destroy")
            self.h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- helpers
    def _dev(self, t, dtype, shape, name, optional=False):
        if t is None:
            if optional:
                return None
            raise PcgrlError(f"{name} is required")
        if not (isinstance(t, torch.Tensor) and t.is_cuda and t.device == self.device):
            raise PcgrlError(f"{name} must be a tensor on {self.device}")
        if t.dtype != dtype or tuple(t.shape) != tuple(shape) or not t.is_contiguous():
            raise PcgrlError(f"{name} must be contiguous {dtype} of shape {tuple(shape)}, "
                             f"got {t.dtype} {tuple(t.shape)}")
        return C.c_void_p(t.data_ptr())

    def new_obs(self):
        return torch.empty(self.obs_shape, dtype=torch.uint8, device=self.device)

    def obs_view(self, obs):
        """The observations proper inside an `obs` buffer (leading slot dimensions allowed): the
        [..., batch, C, ow, ow] one-hot cells as a strided view, or the [..., batch, bytes] packed
        rows, without the bytes a pitch adds after each level."""
        if self.obs_stride == self.obs_bytes and self.cfg.obs_format == 0:
            return obs
        rows = obs[..., :self.obs_bytes]
        if self.cfg.obs_format != 0:
            return rows
        lead = tuple(obs.shape[:-2])
        strides = tuple(obs.stride()[:-2])
        _, Cc, ow, _ = self.onehot_shape
        return rows.as_strided(lead + (self.B, Cc, ow, ow), strides + (self.obs_stride, ow * ow, ow, 1),
                               obs.storage_offset())

    def _st(self):
        return C.c_void_p(_stream_ptr(self.device))

    # -- the C entry points
    def pcgrl_reset(self, seed: int, obs=None):
        o = self._dev(obs, torch.uint8, self.obs_shape, "obs", optional=True)
        _check(self.L.pcgrl_reset(self.h, C.c_uint64(seed), o, self._st()), "pcgrl_reset")

    def pcgrl_step(self, actions, obs=None, reward=None, done=None):
        a = self._dev(actions, torch.int32, (self.B,), "actions")
        o = self._dev(obs, torch.uint8, self.obs_shape, "obs", optional=True)
        r = self._dev(reward, torch.float32, (self.B,), "reward", optional=True)
        d = self._dev(done, torch.uint8, (self.B,), "done", optional=True)
        _check(self.L.pcgrl_step(self.h, a, o, r, d, self._st()), "pcgrl_step")

    def pcgrl_rollout(self, actions, obs=None, reward=None, done=None):
        """actions [T, B]; obs [slots, B, C, ow, ow] (slots <= T); reward / done [T, B]."""
        if not isinstance(actions, torch.Tensor) or actions.dim() != 2:
            raise PcgrlError("actions must be a [T, batch] tensor")
        T = actions.shape[0]
        a = self._dev(actions, torch.int32, (T, self.B), "actions")
        slots = 1
        o = None
        if obs is not None:
            slots = obs.shape[0] if obs.dim() == len(self.obs_shape) + 1 else 0
            o = self._dev(obs, torch.uint8, (slots,) + tuple(self.obs_shape), "obs")
        r = self._dev(reward, torch.float32, (T, self.B), "reward", optional=True)
        d = self._dev(done, torch.uint8, (T, self.B), "done", optional=True)
        _check(self.L.pcgrl_rollout(self.h, a, T, o, slots, r, d, self._st()), "pcgrl_rollout")

    def pcgrl_metrics(self, out=None):
        if out is None:
            out = torch.empty((self.B, self.M), dtype=torch.int32, device=self.device)
        o = self._dev(out, torch.int32, (self.B, self.M), "out")
        _check(self.L.pcgrl_metrics(self.h, o, self._st()), "pcgrl_metrics")
        return out

    def pcgrl_exact_diameter(self, out=None):
        if out is None:
            out = torch.empty((self.B,), dtype=torch.int32, device=self.device)
        o = self._dev(out, torch.int32, (self.B,), "out")
        _check(self.L.pcgrl_exact_diameter(self.h, o, self._st()), "pcgrl_exact_diameter")
        return out

    def pcgrl_exact_diameter_static(self, out, parts_log2: int = -1):
        o = self._dev(out, torch.int32, (self.B,), "out")
        _check(self.L.pcgrl_exact_diameter_static(self.h, o, parts_log2, self._st()), "pcgrl_exact_diameter_static")
        return out

    UNPACK_TYPES = {torch.uint8: 0, torch.float16: 1, torch.bfloat16: 2, torch.float32: 3}

    def pcgrl_unpack_obs(self, packed, out=None, dtype=torch.uint8):
        """Bit-packed observations [batch, stride] -> one-hot [batch, C, ow, ow] of `dtype`."""
        pk = self._dev(packed, torch.uint8, self.obs_shape, "packed")
        if out is None:
            out = torch.empty(self.onehot_shape, dtype=dtype, device=self.device)
        if out.dtype not in self.UNPACK_TYPES:
            raise PcgrlError(f"cannot unpack into {out.dtype}")
        o = self._dev(out, out.dtype, self.onehot_shape, "out")
        _check(self.L.pcgrl_unpack_obs(self.h, pk, o, self.UNPACK_TYPES[out.dtype], self._st()), "pcgrl_unpack_obs")
        return out

    def pcgrl_observe(self, obs=None):
        if obs is None:
            obs = self.new_obs()
        o = self._dev(obs, torch.uint8, self.obs_shape, "obs")
        _check(self.L.pcgrl_observe(self.h, o, self._st()), "pcgrl_observe")
        return obs

    def pcgrl_get_state(self):
        dev = self.device
        tiles = torch.empty((self.B, self.Hm, self.Wm), dtype=torch.int8, device=dev)
        frozen = torch.empty((self.B, self.Hm, self.Wm), dtype=torch.uint8, device=dev)
        hw = torch.empty((self.B, 2), dtype=torch.int16, device=dev)
        pos = torch.empty((self.B, 2), dtype=torch.int16, device=dev)
        ctr = torch.empty((self.B, 3), dtype=torch.int32, device=dev)
        _check(self.L.pcgrl_get_state(self.h, C.c_void_p(tiles.data_ptr()), C.c_void_p(frozen.data_ptr()),
                                      C.c_void_p(hw.data_ptr()), C.c_void_p(pos.data_ptr()),
                                      C.c_void_p(ctr.data_ptr()), self._st()), "pcgrl_get_state")
        return dict(tiles=tiles, frozen=frozen, hw=hw, pos=pos, counters=ctr)

    def pcgrl_set_state(self, tiles, frozen, hw, pos):
        t = self._dev(tiles, torch.int8, (self.B, self.Hm, self.Wm), "tiles")
        f = self._dev(frozen, torch.uint8, (self.B, self.Hm, self.Wm), "frozen", optional=True)
        s = self._dev(hw, torch.int16, (self.B, 2), "hw")
        q = self._dev(pos, torch.int16, (self.B, 2), "pos")
        _check(self.L.pcgrl_set_state(self.h, t, f, s, q, self._st()), "pcgrl_set_state")

    def pcgrl_set_targets(self, targets):
        t = self._dev(targets, torch.int32, (self.B, self.M, 2), "targets")
        _check(self.L.pcgrl_set_targets(self.h, t, self._st()), "pcgrl_set_targets")

    def pcgrl_get_targets(self, out=None):
        if out is None:
            out = torch.empty((self.B, self.M, 2), dtype=torch.int32, device=self.device)
        o = self._dev(out, torch.int32, (self.B, self.M, 2), "out")
        _check(self.L.pcgrl_get_targets(self.h, o, self._st()), "pcgrl_get_targets")
        return out

    def pcgrl_bad_action_count(self) -> int:
        n = C.c_uint64(0)
        _check(self.L.pcgrl_bad_action_count(self.h, C.byref(n), self._st()), "pcgrl_bad_action_count")
        return n.value
