"""ctypes binding of ``libmv.so``: the same calls as ``include/mv.h``, argument marshalling only.

Every step of the render path runs in the HIP kernels behind the C ABI; there is no Python or CPU
fallback.  If the library has not been built, loading fails with an error that says how to build
it.  PyTorch is used by callers only to own device memory and streams: tensors are passed here as
raw device pointers (``tensor.data_ptr()``) and the stream as ``torch.cuda.current_stream().cuda_stream``.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

_PKG_DIR = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG_DIR, "libmv.so")

MV_OK, MV_ERR_ARG, MV_ERR_STATE, MV_ERR_RANGE, MV_ERR_CAPACITY, MV_ERR_HIP = 0, -1, -2, -3, -4, -5
FACE_INSIDE, FACE_MISS = 6, 255

EXPORTS = ("mv_default_config", "mv_create_batch", "mv_upload_worlds", "mv_update_voxels", "mv_set_cameras",
           "mv_render_batch", "mv_set_active", "mv_draw_bars", "mv_draw_overlay", "mv_step", "mv_host_alloc", "mv_host_free",
           "mv_fetch_observations", "mv_destroy", "mv_last_error", "mv_debug_occupancy", "mv_debug_camera_records",
           "mv_debug_set_staged_layers", "mv_debug_launch_shape", "mv_render_worlds_noalloc", "mv_move_voxels")
NOALLOC_SCRATCH_BYTES = 8 << 20


class MvConfig(C.Structure):
    """Mirror of ``mv_config``."""
    _fields_ = [("num_envs", C.c_int32), ("agents_per_env", C.c_int32),
                ("grid_x", C.c_int32), ("grid_y", C.c_int32), ("grid_z", C.c_int32),
                ("width", C.c_int32), ("height", C.c_int32), ("hfov_rad", C.c_float),
                ("num_materials", C.c_int32), ("light_dir", C.c_float * 3),
                ("ambient", C.c_float), ("diffuse", C.c_float), ("sky_rgb", C.c_uint8 * 3),
                ("coarse_level", C.c_uint8), ("device", C.c_int32), ("tiles_per_block", C.c_int32)]


class MvBar(C.Structure):
    """Mirror of ``mv_bar``."""
    _fields_ = [("x", C.c_int32), ("y", C.c_int32), ("width", C.c_int32), ("height", C.c_int32),
                ("fill_rgb", C.c_uint8 * 3), ("empty_rgb", C.c_uint8 * 3), ("reserved", C.c_uint8 * 2)]


class MvRect(C.Structure):
    """Mirror of ``mv_rect``."""
    _fields_ = [("x", C.c_int32), ("y", C.c_int32), ("width", C.c_int32), ("height", C.c_int32),
                ("rgb", C.c_uint8 * 3), ("kind", C.c_uint8), ("rest_rgb", C.c_uint8 * 3), ("value_index", C.c_uint8)]


RECT_SOLID, RECT_GAUGE_RIGHT, RECT_GAUGE_UP = 0, 1, 2
SRC_DEVICE_BORROWED = 2


class MvLaunchShape(C.Structure):
    """Mirror of ``mv_launch_shape``."""
    _fields_ = [(name, C.c_int32) for name in ("lds_bytes", "threads", "tiles_x", "tiles_per_obs", "tiles_per_block",
                                               "blocks_per_obs", "tiles_per_block_tail", "blocks_per_obs_tail",
                                               "num_obs", "obs_per_xcd", "obs_body_per_xcd")] + \
               [("blocks_per_xcd", C.c_uint32)]


class MvStepInputs(C.Structure):
    """Mirror of ``mv_step_inputs``."""
    _fields_ = [("num_edits", C.c_int32), ("edit_env", C.c_void_p), ("edit_voxel", C.c_void_p),
                ("edit_material", C.c_void_p), ("cams", C.c_void_p), ("self_voxel", C.c_void_p),
                ("done", C.c_void_p), ("bar_fraction", C.c_void_p), ("bar", C.POINTER(MvBar)),
                ("overlay", C.POINTER(MvRect)), ("num_overlay", C.c_int32), ("overlay_values_per_obs", C.c_int32),
                ("overlay_values", C.c_void_p)]


class MvError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"mv error {code}: {message}")
        self.code = code


_lib = None


def load_library():
    """Load ``libmv.so`` (built by ``python -m paper_2107_08170_amd.build``); fails loudly if absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2107_08170_amd.build` "
                          "(there is no CPU fallback)")
    lib = C.CDLL(LIB_PATH)
    vp = C.c_void_p
    lib.mv_default_config.argtypes = [C.POINTER(MvConfig)]
    lib.mv_default_config.restype = None
    lib.mv_create_batch.argtypes = [C.POINTER(MvConfig), C.POINTER(vp)]
    lib.mv_upload_worlds.argtypes = [vp, C.c_int32, C.c_int32, vp, vp, C.c_int32, vp]
    lib.mv_update_voxels.argtypes = [vp, C.c_int32, vp, vp, vp, C.c_int32, vp]
    lib.mv_move_voxels.argtypes = [vp, C.c_int32, vp, vp, vp, vp, C.c_int32, vp]
    lib.mv_set_cameras.argtypes = [vp, vp, vp, C.c_int32, vp]
    lib.mv_render_batch.argtypes = [vp, vp, vp, vp, vp, vp, vp]
    lib.mv_set_active.argtypes = [vp, vp, C.c_int32, vp]
    lib.mv_draw_bars.argtypes = [vp, vp, vp, C.POINTER(MvBar), C.c_int32, vp]
    lib.mv_draw_overlay.argtypes = [vp, vp, C.POINTER(MvRect), C.c_int32, vp, C.c_int32, C.c_int32, vp]
    lib.mv_step.argtypes = [vp, C.POINTER(MvStepInputs), vp, vp, vp]
    lib.mv_debug_launch_shape.argtypes = [C.POINTER(MvConfig), C.c_int32, C.POINTER(MvLaunchShape)]
    lib.mv_host_alloc.argtypes = [C.POINTER(vp), C.c_size_t]
    lib.mv_host_free.argtypes = [vp]
    lib.mv_host_free.restype = None
    lib.mv_fetch_observations.argtypes = [vp, vp, vp, C.c_int32, C.c_int32, vp, vp, vp]
    lib.mv_destroy.argtypes = [vp]
    lib.mv_destroy.restype = None
    lib.mv_last_error.restype = C.c_char_p
    lib.mv_debug_occupancy.argtypes = [vp, C.c_int32, C.POINTER(vp), C.POINTER(C.c_int32), C.POINTER(vp),
                                       C.POINTER(C.c_int32), C.POINTER(vp)]
    lib.mv_debug_camera_records.argtypes = [vp, C.POINTER(vp)]
    lib.mv_debug_set_staged_layers.argtypes = [vp, C.c_int32]
    lib.mv_render_worlds_noalloc.argtypes = [C.POINTER(MvConfig), vp, vp, vp, vp, vp, vp, vp]
    _lib = lib
    return lib


def _check(rc: int) -> None:
    if rc != MV_OK:
        raise MvError(rc, load_library().mv_last_error().decode("utf-8", "replace"))


def default_config() -> MvConfig:
    cfg = MvConfig()
    load_library().mv_default_config(C.byref(cfg))
    return cfg


def _as_ptr(x) -> Optional[int]:
    """Raw address of a torch tensor, a NumPy array, an int, or None."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    if hasattr(x, "data_ptr"):
        return x.data_ptr()
    if hasattr(x, "ctypes"):
        return x.ctypes.data
    raise TypeError(f"cannot take the address of {type(x)!r}")


def _is_device(x) -> bool:
    return bool(getattr(x, "is_cuda", False))


def make_config(num_envs: int, agents_per_env: int, grid: Sequence[int], num_materials: int,
                width: int = 128, height: int = 72, hfov_rad: Optional[float] = None,
                light_dir: Optional[Sequence[float]] = None, ambient: Optional[float] = None,
                diffuse: Optional[float] = None, sky_rgb: Optional[Sequence[int]] = None,
                device: int = 0, tiles_per_block: int = 0, coarse_level: int = 0) -> MvConfig:
    """``mv_default_config`` with the given fields filled in."""
    cfg = default_config()
    cfg.num_envs, cfg.agents_per_env = num_envs, agents_per_env
    cfg.grid_x, cfg.grid_y, cfg.grid_z = (int(g) for g in grid)
    cfg.width, cfg.height = width, height
    cfg.num_materials = num_materials
    if hfov_rad is not None:
        cfg.hfov_rad = hfov_rad
    if light_dir is not None:
        cfg.light_dir[:] = [float(v) for v in light_dir]
    if ambient is not None:
        cfg.ambient = ambient
    if diffuse is not None:
        cfg.diffuse = diffuse
    if sky_rgb is not None:
        cfg.sky_rgb[:] = [int(v) for v in sky_rgb]
    cfg.device = device
    cfg.tiles_per_block = tiles_per_block
    cfg.coarse_level = coarse_level
    return cfg


def render_worlds_noalloc(cfg: MvConfig, voxels, palette, cams, self_voxel, rgb, depth, stream: int = 0) -> None:
    """``mv_render_worlds_noalloc``: pack, cameras and render in one call that allocates nothing; all array
    arguments are device tensors (or raw device addresses)."""
    _check(load_library().mv_render_worlds_noalloc(C.byref(cfg), _as_ptr(voxels), _as_ptr(palette), _as_ptr(cams),
                                                   _as_ptr(self_voxel), _as_ptr(rgb), _as_ptr(depth), stream))


def _pack_rects(rects):
    """A ctypes array of ``mv_rect`` from (x, y, width, height, rgb, kind, rest_rgb, value_index) tuples."""
    packed = (MvRect * max(len(rects), 1))()
    for k, (x, y, width, height, colour, kind, rest, value_index) in enumerate(rects):
        q = packed[k]
        q.x, q.y, q.width, q.height, q.kind, q.value_index = x, y, width, height, kind, value_index
        q.rgb[:] = [int(v) for v in colour]
        q.rest_rgb[:] = [int(v) for v in rest]
    return packed


def launch_shape(cfg: MvConfig, staged_layers: int = 0) -> MvLaunchShape:
    """The launch layout of a render of ``cfg`` (host arithmetic only, no GPU needed)."""
    shape = MvLaunchShape()
    _check(load_library().mv_debug_launch_shape(C.byref(cfg), staged_layers, C.byref(shape)))
    return shape


class PinnedBuffer:
    """Page-locked host memory from ``mv_host_alloc``; ``array(dtype, shape)`` views it as a NumPy array."""

    def __init__(self, nbytes: int):
        ptr = C.c_void_p()
        _check(load_library().mv_host_alloc(C.byref(ptr), nbytes))
        self.address, self.nbytes = ptr.value, nbytes

    def array(self, dtype, shape):
        import numpy as np
        buf = (C.c_uint8 * self.nbytes).from_address(self.address)
        return np.frombuffer(buf, dtype=dtype, count=int(np.prod(shape))).reshape(shape)

    def close(self) -> None:
        if self.address:
            load_library().mv_host_free(self.address)
            self.address = 0


class Batch:
    """N environments x A agent cameras on one GPU (thin wrapper over the ``mv_batch*`` handle)."""

    def __init__(self, num_envs: int, agents_per_env: int, grid: Sequence[int], num_materials: int,
                 width: int = 128, height: int = 72, hfov_rad: Optional[float] = None,
                 light_dir: Optional[Sequence[float]] = None, ambient: Optional[float] = None,
                 diffuse: Optional[float] = None, sky_rgb: Optional[Sequence[int]] = None,
                 device: int = 0, tiles_per_block: int = 0, coarse_level: int = 0):
        lib = load_library()
        cfg = make_config(num_envs, agents_per_env, grid, num_materials, width, height, hfov_rad, light_dir, ambient,
                          diffuse, sky_rgb, device, tiles_per_block, coarse_level)
        self.cfg = cfg
        self._h = C.c_void_p()
        _check(lib.mv_create_batch(C.byref(cfg), C.byref(self._h)))
        self.num_obs = num_envs * agents_per_env

    def upload_worlds(self, voxels, palette=None, first_env: int = 0, count: Optional[int] = None,
                      stream: int = 0, borrow: bool = False) -> None:
        """``voxels`` u8[count,Z,Y,X] and ``palette`` u8[count,M+1,3]: both torch CUDA tensors or both
        host arrays (NumPy / CPU tensors).  ``borrow``: the device tensor of all environments is not copied; the
        batch reads material ids from it until the next upload (the caller keeps it alive and unchanged)."""
        if count is None:
            count = int(voxels.shape[0])
        dev = _is_device(voxels)
        if palette is not None and _is_device(palette) != dev:
            raise ValueError("voxels and palette must live in the same memory space")
        if borrow and not dev:
            raise ValueError("only a device tensor can be borrowed")
        _check(load_library().mv_upload_worlds(self._h, first_env, count, _as_ptr(voxels), _as_ptr(palette),
                                               SRC_DEVICE_BORROWED if borrow else (1 if dev else 0), stream))

    def update_voxels(self, env, voxel_index, material, stream: int = 0) -> None:
        """Sparse edits: ``env`` i32[count], ``voxel_index`` i32[count], ``material`` u8[count], all three
        torch CUDA tensors or all three host arrays."""
        count = int(env.shape[0])
        dev = _is_device(env)
        if _is_device(voxel_index) != dev or _is_device(material) != dev:
            raise ValueError("env, voxel_index and material must live in the same memory space")
        _check(load_library().mv_update_voxels(self._h, count, _as_ptr(env), _as_ptr(voxel_index), _as_ptr(material),
                                               1 if dev else 0, stream))

    def move_voxels(self, env, from_voxel, to_voxel, material, stream: int = 0) -> None:
        """Objects that moved: ``env``, ``from_voxel``, ``to_voxel`` i32[count] and ``material`` u8[count], all four torch
        CUDA tensors or all four host arrays."""
        count = int(env.shape[0])
        dev = _is_device(env)
        if any(_is_device(a) != dev for a in (from_voxel, to_voxel, material)):
            raise ValueError("env, from_voxel, to_voxel and material must live in the same memory space")
        _check(load_library().mv_move_voxels(self._h, count, _as_ptr(env), _as_ptr(from_voxel), _as_ptr(to_voxel),
                                             _as_ptr(material), 1 if dev else 0, stream))

    def set_cameras(self, cams, self_voxel=None, stream: int = 0) -> None:
        dev = _is_device(cams)
        if self_voxel is not None and _is_device(self_voxel) != dev:
            raise ValueError("cams and self_voxel must live in the same memory space")
        _check(load_library().mv_set_cameras(self._h, _as_ptr(cams), _as_ptr(self_voxel), 1 if dev else 0, stream))

    def render(self, rgb, depth, aux_material=None, aux_hit_index=None, aux_face=None, stream: int = 0) -> None:
        _check(load_library().mv_render_batch(self._h, _as_ptr(rgb), _as_ptr(depth), _as_ptr(aux_material),
                                              _as_ptr(aux_hit_index), _as_ptr(aux_face), stream))

    def set_active(self, active, stream: int = 0) -> None:
        """``active`` u8[N] (non-zero = render) as a torch CUDA tensor or a host array; None = all."""
        _check(load_library().mv_set_active(self._h, _as_ptr(active), 1 if _is_device(active) else 0, stream))

    def draw_bars(self, rgb, fraction, x: int, y: int, width: int, height: int, fill_rgb, empty_rgb,
                  stream: int = 0) -> None:
        bar = MvBar()
        bar.x, bar.y, bar.width, bar.height = x, y, width, height
        bar.fill_rgb[:] = [int(v) for v in fill_rgb]
        bar.empty_rgb[:] = [int(v) for v in empty_rgb]
        _check(load_library().mv_draw_bars(self._h, _as_ptr(rgb), _as_ptr(fraction), C.byref(bar),
                                           1 if _is_device(fraction) else 0, stream))

    def draw_overlay(self, rgb, rects, values=None, stream: int = 0) -> None:
        """``rects``: a sequence of (x, y, width, height, rgb, kind, rest_rgb, value_index), painted in this order;
        ``values``: f32[N*A, k] as a torch CUDA tensor or a host array, or None when no primitive is a gauge."""
        packed = _pack_rects(rects)
        per_obs = 0 if values is None else int(values.shape[1])
        _check(load_library().mv_draw_overlay(self._h, _as_ptr(rgb), packed, len(rects), _as_ptr(values), per_obs,
                                              1 if values is not None and _is_device(values) else 0, stream))

    def step(self, cams, rgb, depth, edits=None, self_voxel=None, done=None, bar_fraction=None, bar=None,
             overlay=None, overlay_values=None, stream: int = 0) -> None:
        """One whole step from device tensors: ``edits`` = (env i32[n], voxel i32[n], material u8[n]) or None,
        ``done`` u8[N] or None, ``bar`` = dict(x, y, width, height, fill_rgb, empty_rgb) with ``bar_fraction``
        f32[N*A], ``overlay`` = primitives as for ``draw_overlay`` with ``overlay_values`` f32[N*A, k]."""
        inp = MvStepInputs()
        if edits is not None:
            env, voxel, material = edits
            inp.num_edits = int(env.shape[0])
            inp.edit_env, inp.edit_voxel, inp.edit_material = _as_ptr(env), _as_ptr(voxel), _as_ptr(material)
        inp.cams = _as_ptr(cams)
        inp.self_voxel = _as_ptr(self_voxel)
        inp.done = _as_ptr(done)
        inp.bar_fraction = _as_ptr(bar_fraction)
        c_bar = None
        if bar is not None:
            c_bar = MvBar()
            c_bar.x, c_bar.y, c_bar.width, c_bar.height = bar["x"], bar["y"], bar["width"], bar["height"]
            c_bar.fill_rgb[:] = [int(v) for v in bar["fill_rgb"]]
            c_bar.empty_rgb[:] = [int(v) for v in bar["empty_rgb"]]
            inp.bar = C.pointer(c_bar)
        if overlay:
            packed = _pack_rects(overlay)
            inp.overlay, inp.num_overlay = packed, len(overlay)
            if overlay_values is not None:
                inp.overlay_values, inp.overlay_values_per_obs = _as_ptr(overlay_values), int(overlay_values.shape[1])
        _check(load_library().mv_step(self._h, C.byref(inp), _as_ptr(rgb), _as_ptr(depth), stream))

    def fetch_observations(self, rgb_dev, depth_dev, first_obs: int, count: int, rgb_host, depth_host,
                           stream: int = 0) -> None:
        """Enqueue the device-to-host copy of a range of observations; host arguments are NumPy arrays,
        ``PinnedBuffer.address`` integers or None."""
        _check(load_library().mv_fetch_observations(self._h, _as_ptr(rgb_dev), _as_ptr(depth_dev), first_obs, count,
                                                    _as_ptr(rgb_host), _as_ptr(depth_host), stream))

    def debug_occupancy(self, env: int):
        """(x_rows_ptr, x_row_words, y_rows_ptr, y_row_words, top_layer_ptr) of one environment."""
        xp, yp, tp = C.c_void_p(), C.c_void_p(), C.c_void_p()
        xw, yw = C.c_int32(), C.c_int32()
        _check(load_library().mv_debug_occupancy(self._h, env, C.byref(xp), C.byref(xw), C.byref(yp), C.byref(yw),
                                                 C.byref(tp)))
        return xp.value, xw.value, yp.value, yw.value, tp.value

    def debug_set_staged_layers(self, layers: int) -> None:
        _check(load_library().mv_debug_set_staged_layers(self._h, layers))

    def debug_camera_records(self) -> int:
        ptr = C.c_void_p()
        _check(load_library().mv_debug_camera_records(self._h, C.byref(ptr)))
        return ptr.value

    def close(self) -> None:
        if getattr(self, "_h", None) is not None and self._h.value:
            load_library().mv_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
