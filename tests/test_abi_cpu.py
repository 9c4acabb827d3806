"""CPU-only checks of the C ABI: the library loads, exports every symbol the header declares, and
rejects bad arguments before touching the GPU.  No compute call is made here."""
import ctypes as C
import os
import re

import pytest

import paper_2107_08170_amd as mv
from paper_2107_08170_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2107_08170_amd import build
        build.build()
    return mv.load_library()


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "mv.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(mv_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = _declared_symbols()
    assert {"mv_create_batch", "mv_upload_worlds", "mv_set_cameras", "mv_render_batch", "mv_destroy"} <= set(names)
    for name in names:
        assert hasattr(lib, name), name
    assert set(names) == set(binding.EXPORTS)


def test_config_struct_layout_matches_header(lib):
    cfg = binding.default_config()
    # ask a C compiler for the header's layout and compare with the ctypes mirror
    import subprocess, tempfile
    fields = [f[0] for f in binding.MvConfig._fields_]
    prog = '#include <stdio.h>\n#include <stddef.h>\n#include "mv.h"\nint main(void){printf("%zu", sizeof(mv_config));' + \
        "".join(f'printf(" %zu", offsetof(mv_config, {f}));' for f in fields) + "return 0;}"
    with tempfile.TemporaryDirectory() as tmp:
        src, exe = os.path.join(tmp, "layout.c"), os.path.join(tmp, "layout")
        open(src, "w").write(prog)
        subprocess.run(["gcc", "-I", os.path.join(ROOT, "include"), src, "-o", exe], check=True)
        numbers = [int(x) for x in subprocess.run([exe], check=True, capture_output=True, text=True).stdout.split()]
    assert numbers[0] == C.sizeof(binding.MvConfig)
    assert numbers[1:] == [getattr(binding.MvConfig, f).offset for f in fields]
    assert (cfg.width, cfg.height) == (128, 72)
    assert abs(cfg.hfov_rad - 1.5707964) < 1e-6
    assert list(cfg.light_dir) == [1.0, 2.0, 3.0] and list(cfg.sky_rgb) == [135, 206, 235]
    assert abs(cfg.ambient - 0.3) < 1e-7 and abs(cfg.diffuse - 0.7) < 1e-7
    assert cfg.device == 0 and cfg.tiles_per_block == 0 and cfg.num_envs == 0


@pytest.mark.parametrize("c_name,mirror", [("mv_bar", "MvBar"), ("mv_rect", "MvRect"), ("mv_step_inputs", "MvStepInputs")])
def test_overlay_struct_layouts_match_header(c_name, mirror):
    import subprocess, tempfile
    cls = getattr(binding, mirror)
    fields = [f[0] for f in cls._fields_]
    prog = '#include <stdio.h>\n#include <stddef.h>\n#include "mv.h"\nint main(void){printf("%zu", sizeof(' + c_name + '));' + \
        "".join(f'printf(" %zu", offsetof({c_name}, {f}));' for f in fields) + "return 0;}"
    with tempfile.TemporaryDirectory() as tmp:
        src, exe = os.path.join(tmp, "layout.c"), os.path.join(tmp, "layout")
        open(src, "w").write(prog)
        subprocess.run(["gcc", "-I", os.path.join(ROOT, "include"), src, "-o", exe], check=True)
        numbers = [int(x) for x in subprocess.run([exe], check=True, capture_output=True, text=True).stdout.split()]
    assert numbers[0] == C.sizeof(cls)
    assert numbers[1:] == [getattr(cls, f).offset for f in fields]


@pytest.mark.parametrize("field,value", [
    ("num_envs", 0), ("agents_per_env", -1), ("grid_x", 0), ("grid_z", -3), ("width", 0), ("height", 20000),
    ("hfov_rad", 0.0), ("hfov_rad", 3.2), ("num_materials", 0), ("num_materials", 256), ("coarse_level", 2),
    ("tiles_per_block", -1), ("device", -1), ("ambient", float("nan")),
])
def test_create_rejects_bad_config_before_any_gpu_call(lib, field, value):
    cfg = binding.default_config()
    cfg.num_envs, cfg.agents_per_env, cfg.num_materials = 2, 1, 4
    cfg.grid_x = cfg.grid_y = cfg.grid_z = 4
    setattr(cfg, field, value)
    handle = C.c_void_p()
    rc = lib.mv_create_batch(C.byref(cfg), C.byref(handle))
    assert rc == binding.MV_ERR_ARG, (field, rc, lib.mv_last_error())
    assert handle.value is None
    assert lib.mv_last_error() != b""


def test_create_rejects_zero_light_and_oversized_grid(lib):
    cfg = binding.default_config()
    cfg.num_envs, cfg.agents_per_env, cfg.num_materials = 1, 1, 4
    cfg.grid_x = cfg.grid_y = cfg.grid_z = 4
    cfg.light_dir[:] = [0.0, 0.0, 0.0]
    handle = C.c_void_p()
    assert lib.mv_create_batch(C.byref(cfg), C.byref(handle)) == binding.MV_ERR_ARG
    cfg.light_dir[:] = [0.0, 0.0, 1.0]
    cfg.grid_x, cfg.grid_y, cfg.grid_z = 256, 256, 64       # 512 KiB of occupancy bits: beyond the LDS plan
    assert lib.mv_create_batch(C.byref(cfg), C.byref(handle)) == binding.MV_ERR_CAPACITY
    assert b"LDS" in lib.mv_last_error()


def test_create_rejects_layers_the_pack_kernel_cannot_hold(lib):
    """256x256x2: only 16 KiB of occupancy bits (fits the render plan), but the pack kernel keeps a whole 64 KiB
    layer per wave in LDS, four waves: beyond a compute unit's 160 KiB.  Must be refused at creation, not fail at
    the first upload."""
    cfg = binding.default_config()
    cfg.num_envs, cfg.agents_per_env, cfg.num_materials = 1, 1, 4
    cfg.grid_x, cfg.grid_y, cfg.grid_z = 256, 256, 2
    handle = C.c_void_p()
    assert lib.mv_create_batch(C.byref(cfg), C.byref(handle)) == binding.MV_ERR_CAPACITY
    assert b"packing" in lib.mv_last_error() and handle.value is None


def test_null_arguments(lib):
    handle = C.c_void_p()
    assert lib.mv_create_batch(None, C.byref(handle)) == binding.MV_ERR_ARG
    assert lib.mv_create_batch(C.byref(binding.default_config()), None) == binding.MV_ERR_ARG
    assert lib.mv_upload_worlds(None, 0, 1, None, None, 0, None) == binding.MV_ERR_ARG
    assert lib.mv_set_cameras(None, None, None, 0, None) == binding.MV_ERR_ARG
    assert lib.mv_render_batch(None, None, None, None, None, None, None) == binding.MV_ERR_ARG
    assert lib.mv_fetch_observations(None, None, None, 0, 1, None, None, None) == binding.MV_ERR_ARG
    assert lib.mv_move_voxels(None, 1, None, None, None, None, 0, None) == binding.MV_ERR_ARG
    assert lib.mv_draw_bars(None, None, None, None, 0, None) == binding.MV_ERR_ARG
    assert lib.mv_draw_overlay(None, None, None, 1, None, 0, 0, None) == binding.MV_ERR_ARG
    assert lib.mv_step(None, None, None, None, None) == binding.MV_ERR_ARG
    assert lib.mv_step(None, C.byref(binding.MvStepInputs()), None, None, None) == binding.MV_ERR_ARG
    assert lib.mv_host_alloc(None, 16) == binding.MV_ERR_ARG
    out = C.c_void_p()
    assert lib.mv_host_alloc(C.byref(out), 0) == binding.MV_ERR_ARG
    lib.mv_host_free(None)                                  # NULL-safe
    lib.mv_destroy(None)                                    # NULL-safe
    lib.mv_default_config(None)


def test_product_package_does_not_touch_the_oracle():
    """The product path must never route through the CPU oracle."""
    pkg = os.path.join(ROOT, "paper_2107_08170_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.lower() or f == "synth.py", f
    synth_text = open(os.path.join(pkg, "synth.py")).read()
    assert "import oracle" not in synth_text and "from oracle" not in synth_text
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith((".py", ".c", ".h")):
            text = open(os.path.join(ROOT, "oracle", f)).read()
            assert "paper_2107_08170_amd" not in text and "mv.h" not in text.replace("mv_oracle.h", ""), f
