"""ctypes front end of the CPU oracle (``oracle/mv_oracle.c`` + ``oracle/mv_definition.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by the smoke check and by the benchmark's
``cpu_baseline`` leg.  The product package never imports this module, and this module never
imports the product package.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libmv_oracle.so")
_SOURCES = ("mv_oracle.c", "mv_definition.c")

FACE_INSIDE = 6
FACE_MISS = 255


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (strict IEEE arithmetic: no contraction, no fast-math)."""
    srcs = [os.path.join(_HERE, s) for s in _SOURCES]
    deps = srcs + [os.path.join(_HERE, "mv_oracle.h")]
    if not force and os.path.exists(_LIB_PATH) and all(
            os.path.getmtime(_LIB_PATH) >= os.path.getmtime(p) for p in deps):
        return _LIB_PATH
    cmd = ["gcc", "-std=c11", "-O2", "-fPIC", "-shared", "-ffp-contract=off", "-fno-fast-math",
           "-Wall", "-Wextra", "-o", _LIB_PATH] + srcs + ["-lm", "-lpthread"]
    subprocess.run(cmd, check=True)
    return _LIB_PATH


class _Config(C.Structure):
    _fields_ = [("num_envs", C.c_int32), ("agents_per_env", C.c_int32),
                ("grid_x", C.c_int32), ("grid_y", C.c_int32), ("grid_z", C.c_int32),
                ("width", C.c_int32), ("height", C.c_int32), ("hfov_rad", C.c_float),
                ("num_materials", C.c_int32), ("light_dir", C.c_float * 3),
                ("ambient", C.c_float), ("diffuse", C.c_float), ("sky_rgb", C.c_uint8 * 3),
                ("pad_", C.c_uint8)]


_lib = None


def _load():
    global _lib
    if _lib is not None:
        return _lib
    other = os.environ.get("MV_ORACLE_LIBRARY")     # another build of the same sources (the sanitizer test's)
    if other:
        _lib = _bind(C.CDLL(other))
        return _lib
    build()
    _lib = _bind(C.CDLL(_LIB_PATH))
    return _lib


class use_library:
    """Context manager: run the front end against another build of the oracle sources (the mutation
    tests compile deliberately broken copies and check that the pins notice)."""

    def __init__(self, path: str):
        self._path = path

    def __enter__(self):
        global _lib
        _load()
        self._saved = _lib
        _lib = _bind(C.CDLL(self._path))
        return self

    def __exit__(self, *exc):
        global _lib
        _lib = self._saved
        return False


def _bind(lib):
    vp = C.c_void_p
    lib.mvo_create.argtypes = [C.POINTER(_Config), C.POINTER(vp)]
    lib.mvo_destroy.argtypes = [vp]
    lib.mvo_destroy.restype = None
    lib.mvo_upload_worlds.argtypes = [vp, C.c_int32, C.c_int32, vp, vp]
    lib.mvo_update_voxels.argtypes = [vp, C.c_int32, vp, vp, vp]
    lib.mvo_set_cameras.argtypes = [vp, vp, vp]
    lib.mvo_render.argtypes = [vp, C.c_int32, C.c_int32] + [vp] * 8 + [C.c_int32]
    lib.mvo_render_pixels.argtypes = [vp, C.c_int64] + [vp] * 11
    lib.mvo_draw_bars.argtypes = [vp, C.c_int32, C.c_int32, vp, vp] + [C.c_int32] * 4 + [vp, vp, vp]
    lib.mvo_draw_overlay.argtypes = [vp, C.c_int32, C.c_int32, vp, vp, C.c_int32, vp, C.c_int32, vp]
    lib.mvo_camera_record.argtypes = [vp, C.c_int32, vp]
    lib.mvo_pixel_ray.argtypes = [vp, C.c_int32, C.c_int32, C.c_int32, vp]
    lib.mvo_face_intensity.argtypes = [vp, vp]
    lib.mvo_quantise.argtypes = [C.c_uint8, C.c_float]
    lib.mvo_quantise.restype = C.c_uint8
    lib.mvd_first_hit_batch.argtypes = [C.c_int32] * 3 + [vp, C.c_int64] + [vp] * 6
    lib.mvd_first_hit_batch.restype = None
    return lib


# layout of mvo_rect (24 bytes, no padding)
RECT_DTYPE = np.dtype([("x", np.int32), ("y", np.int32), ("width", np.int32), ("height", np.int32),
                       ("rgb", np.uint8, 3), ("kind", np.uint8), ("rest_rgb", np.uint8, 3), ("value_index", np.uint8)])
assert RECT_DTYPE.itemsize == 24


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


@dataclass
class Rendered:
    rgb: np.ndarray           # u8 [n,H,W,3]
    depth: np.ndarray         # f32 [n,H,W]
    material: np.ndarray      # u8 [n,H,W]
    hit_index: np.ndarray     # i32 [n,H,W]
    face: np.ndarray          # u8 [n,H,W]
    steps: np.ndarray         # i32 [n,H,W]
    edge_margin: np.ndarray   # f64 [n,H,W]
    t: np.ndarray             # f64 [n,H,W]


DEFAULT_LIGHT = (1.0, 2.0, 3.0)
DEFAULT_SKY = (135, 206, 235)


class OracleBatch:
    """Same five operations as the GPU library, host arrays in and out."""

    def __init__(self, num_envs: int, agents_per_env: int, grid: Sequence[int], width: int,
                 height: int, num_materials: int, hfov_rad: float = float(np.float32(np.pi / 2)),
                 light_dir: Sequence[float] = DEFAULT_LIGHT, ambient: float = 0.30,
                 diffuse: float = 0.70, sky_rgb: Sequence[int] = DEFAULT_SKY):
        lib = _load()
        cfg = _Config()
        cfg.num_envs, cfg.agents_per_env = num_envs, agents_per_env
        cfg.grid_x, cfg.grid_y, cfg.grid_z = grid
        cfg.width, cfg.height = width, height
        cfg.hfov_rad = hfov_rad
        cfg.num_materials = num_materials
        cfg.light_dir[:] = [float(v) for v in light_dir]
        cfg.ambient, cfg.diffuse = ambient, diffuse
        cfg.sky_rgb[:] = [int(v) for v in sky_rgb]
        self._h = C.c_void_p()
        rc = lib.mvo_create(C.byref(cfg), C.byref(self._h))
        if rc != 0:
            raise ValueError(f"mvo_create failed ({rc})")
        self.N, self.A = num_envs, agents_per_env
        self.grid = tuple(int(g) for g in grid)
        self.W, self.H, self.M = width, height, num_materials

    def close(self):
        if getattr(self, "_h", None):
            _load().mvo_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:       # interpreter shutdown: module globals may already be gone
            pass

    def upload_worlds(self, voxels: np.ndarray, palette: Optional[np.ndarray], first_env: int = 0):
        X, Y, Z = self.grid
        voxels = np.ascontiguousarray(voxels, dtype=np.uint8)
        assert voxels.shape[1:] == (Z, Y, X), voxels.shape
        if palette is not None:
            palette = np.ascontiguousarray(palette, dtype=np.uint8)
            assert palette.shape == (voxels.shape[0], self.M + 1, 3), palette.shape
        rc = _load().mvo_upload_worlds(self._h, first_env, voxels.shape[0], _ptr(voxels), _ptr(palette))
        if rc != 0:
            raise ValueError(f"mvo_upload_worlds failed ({rc})")

    def update_voxels(self, env: np.ndarray, voxel_index: np.ndarray, material: np.ndarray):
        env = np.ascontiguousarray(env, dtype=np.int32)
        voxel_index = np.ascontiguousarray(voxel_index, dtype=np.int32)
        material = np.ascontiguousarray(material, dtype=np.uint8)
        assert env.shape == voxel_index.shape == material.shape and env.ndim == 1
        rc = _load().mvo_update_voxels(self._h, env.shape[0], _ptr(env), _ptr(voxel_index), _ptr(material))
        if rc != 0:
            raise ValueError(f"mvo_update_voxels failed ({rc})")

    def set_cameras(self, cams: np.ndarray, self_voxel: Optional[np.ndarray] = None):
        cams = np.ascontiguousarray(cams, dtype=np.float32)
        assert cams.shape == (self.N * self.A, 5), cams.shape
        if self_voxel is not None:
            self_voxel = np.ascontiguousarray(self_voxel, dtype=np.int32)
            assert self_voxel.shape == (self.N * self.A,)
        rc = _load().mvo_set_cameras(self._h, _ptr(cams), _ptr(self_voxel))
        if rc != 0:
            raise ValueError(f"mvo_set_cameras failed ({rc})")

    def render(self, first_obs: int = 0, count: Optional[int] = None, threads: int = 1,
               side_channels=True) -> Rendered:
        """``side_channels``: True = steps, edge margin and exact t; "steps" = the step counter only; False = none."""
        n = self.N * self.A - first_obs if count is None else count
        H, W = self.H, self.W
        all_channels = side_channels is True
        out = Rendered(np.empty((n, H, W, 3), np.uint8), np.empty((n, H, W), np.float32),
                       np.empty((n, H, W), np.uint8), np.empty((n, H, W), np.int32),
                       np.empty((n, H, W), np.uint8),
                       np.empty((n, H, W), np.int32) if side_channels else None,
                       np.empty((n, H, W), np.float64) if all_channels else None,
                       np.empty((n, H, W), np.float64) if all_channels else None)
        rc = _load().mvo_render(self._h, first_obs, n, _ptr(out.rgb), _ptr(out.depth),
                                _ptr(out.material), _ptr(out.hit_index), _ptr(out.face),
                                _ptr(out.steps), _ptr(out.edge_margin), _ptr(out.t), threads)
        if rc != 0:
            raise ValueError(f"mvo_render failed ({rc})")
        return out

    def render_pixels(self, obs: np.ndarray, row: np.ndarray, col: np.ndarray) -> Rendered:
        obs = np.ascontiguousarray(obs, dtype=np.int32)
        row = np.ascontiguousarray(row, dtype=np.int32)
        col = np.ascontiguousarray(col, dtype=np.int32)
        n = obs.shape[0]
        out = Rendered(np.empty((n, 3), np.uint8), np.empty(n, np.float32), np.empty(n, np.uint8),
                       np.empty(n, np.int32), np.empty(n, np.uint8), np.empty(n, np.int32),
                       np.empty(n, np.float64), np.empty(n, np.float64))
        rc = _load().mvo_render_pixels(self._h, n, _ptr(obs), _ptr(row), _ptr(col), _ptr(out.rgb),
                                       _ptr(out.depth), _ptr(out.material), _ptr(out.hit_index),
                                       _ptr(out.face), _ptr(out.steps), _ptr(out.edge_margin),
                                       _ptr(out.t))
        if rc != 0:
            raise ValueError(f"mvo_render_pixels failed ({rc})")
        return out

    def draw_bars(self, rgb: np.ndarray, fraction: np.ndarray, x: int, y: int, width: int, height: int,
                  fill_rgb, empty_rgb, first_obs: int = 0, active: Optional[np.ndarray] = None):
        """Paint the indicator bar into ``rgb`` (u8[count,H,W,3], modified in place)."""
        assert rgb.dtype == np.uint8 and rgb.flags.c_contiguous and rgb.shape[1:] == (self.H, self.W, 3)
        fraction = np.ascontiguousarray(fraction, dtype=np.float32)
        assert fraction.shape == (rgb.shape[0],)
        fill = np.asarray(fill_rgb, np.uint8)
        empty = np.asarray(empty_rgb, np.uint8)
        if active is not None:
            active = np.ascontiguousarray(active, dtype=np.uint8)
            assert active.shape == (self.N,)
        rc = _load().mvo_draw_bars(self._h, first_obs, rgb.shape[0], _ptr(rgb), _ptr(fraction), x, y, width, height,
                                   _ptr(fill), _ptr(empty), _ptr(active))
        if rc != 0:
            raise ValueError(f"mvo_draw_bars failed ({rc})")

    def draw_overlay(self, rgb: np.ndarray, rects, values: Optional[np.ndarray] = None, first_obs: int = 0,
                     active: Optional[np.ndarray] = None):
        """Paint a list of primitives into ``rgb`` (u8[count,H,W,3], modified in place).  ``rects`` is a sequence of
        (x, y, width, height, rgb, kind, rest_rgb, value_index); ``values`` is f32[count, values_per_obs]."""
        assert rgb.dtype == np.uint8 and rgb.flags.c_contiguous and rgb.shape[1:] == (self.H, self.W, 3)
        packed = np.zeros(len(rects), RECT_DTYPE)
        for k, (x, y, w, h, colour, kind, rest, value_index) in enumerate(rects):
            packed[k] = (x, y, w, h, tuple(colour), kind, tuple(rest), value_index)
        per_obs = 0
        if values is not None:
            values = np.ascontiguousarray(values, dtype=np.float32)
            assert values.ndim == 2 and values.shape[0] == rgb.shape[0]
            per_obs = values.shape[1]
        if active is not None:
            active = np.ascontiguousarray(active, dtype=np.uint8)
            assert active.shape == (self.N,)
        rc = _load().mvo_draw_overlay(self._h, first_obs, rgb.shape[0], _ptr(rgb), _ptr(packed), len(rects),
                                      _ptr(values), per_obs, _ptr(active))
        if rc != 0:
            raise ValueError(f"mvo_draw_overlay failed ({rc})")

    def camera_record(self, obs: int) -> np.ndarray:
        rec = np.empty(12, np.float32)
        rc = _load().mvo_camera_record(self._h, obs, _ptr(rec))
        if rc != 0:
            raise ValueError(f"mvo_camera_record failed ({rc})")
        return rec

    def pixel_rays(self, obs: int) -> np.ndarray:
        """f32[H,W,3] ray directions of one observation."""
        out = np.empty((self.H, self.W, 3), np.float32)
        d = np.empty(3, np.float32)
        lib = _load()
        for r in range(self.H):
            for c in range(self.W):
                rc = lib.mvo_pixel_ray(self._h, obs, r, c, _ptr(d))
                if rc != 0:
                    raise ValueError(f"mvo_pixel_ray failed ({rc})")
                out[r, c] = d
        return out

    def face_intensity(self) -> np.ndarray:
        out = np.empty(7, np.float32)
        _load().mvo_face_intensity(self._h, _ptr(out))
        return out


def quantise(palette_value: int, intensity: float) -> int:
    return int(_load().mvo_quantise(int(palette_value), float(np.float32(intensity))))


def definition_first_hit(grid: Sequence[int], vox: np.ndarray, P: np.ndarray, d: np.ndarray,
                         self_voxel: Optional[np.ndarray] = None):
    """Definition D on one grid for n rays: returns (hit_index i32[n], face i32[n], t f64[n])."""
    X, Y, Z = (int(g) for g in grid)
    vox = np.ascontiguousarray(vox, dtype=np.uint8)
    assert vox.shape == (Z, Y, X)
    P = np.ascontiguousarray(P, dtype=np.float64).reshape(-1, 3)
    d = np.ascontiguousarray(d, dtype=np.float64).reshape(-1, 3)
    n = P.shape[0]
    assert d.shape[0] == n
    if self_voxel is not None:
        self_voxel = np.ascontiguousarray(self_voxel, dtype=np.int32)
    hit = np.empty(n, np.int32)
    face = np.empty(n, np.int32)
    t = np.empty(n, np.float64)
    _load().mvd_first_hit_batch(X, Y, Z, _ptr(vox), n, _ptr(P), _ptr(d), _ptr(self_voxel),
                                _ptr(hit), _ptr(face), _ptr(t))
    return hit, face, t
