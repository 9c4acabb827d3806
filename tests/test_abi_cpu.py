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


@pytest.mark.parametrize("c_name,mirror", [("mv_bar", "MvBar"), ("mv_rect", "MvRect"), ("mv_step_inputs", "MvStepInputs"),
                                           ("mv_launch_shape", "MvLaunchShape")])
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


# ------------------------------------------------------------------------------------------ launch layout (host logic)
def _work_list(shape):
    """Replays the documented mapping of workgroups to (observation, tile range): for every workgroup of the launch
    either nothing (a surplus workgroup) or one strip."""
    out = []
    for b in range(8 * shape.blocks_per_xcd):
        xcd, seq = b % 8, b // 8
        body = shape.obs_body_per_xcd * shape.blocks_per_obs
        if seq < body:
            local, part, tpb, strips = seq // shape.blocks_per_obs, seq % shape.blocks_per_obs, shape.tiles_per_block, shape.blocks_per_obs
        else:
            s2 = seq - body
            local, part = shape.obs_body_per_xcd + s2 // shape.blocks_per_obs_tail, s2 % shape.blocks_per_obs_tail
            tpb, strips = shape.tiles_per_block_tail, shape.blocks_per_obs_tail
            if local >= shape.obs_per_xcd:
                continue
        obs = xcd * shape.obs_per_xcd + local
        if obs >= shape.num_obs:
            continue
        begin = part * tpb
        out.append((obs, begin, min(begin + tpb, shape.tiles_per_obs), strips))
    return out


@pytest.mark.parametrize("envs,agents,grid,image,staged", [
    (4, 1, (16, 16, 8), (128, 72), 0), (256, 4, (40, 40, 16), (128, 72), 0), (4096, 2, (40, 40, 16), (128, 72), 10),
    (1024, 4, (40, 40, 16), (128, 72), 10), (2048, 4, (64, 64, 32), (256, 144), 16), (1, 1, (1, 1, 1), (1, 1), 0),
    (3, 5, (7, 5, 3), (33, 19), 0), (2, 1, (40, 40, 16), (1920, 1080), 0), (2, 1, (40, 40, 16), (16384, 8), 0),
    (1000, 3, (64, 64, 6), (130, 70), 2), (17, 1, (128, 128, 32), (64, 40), 0), (9, 2, (96, 96, 16), (128, 72), 0),
])
def test_every_tile_of_every_observation_belongs_to_exactly_one_workgroup(lib, envs, agents, grid, image, staged):
    """The launch layout, computed on the host: the strips of the work list cover every tile of every observation once,
    nothing else and nothing twice; the workgroup fits the compute unit; the image tiling covers the image."""
    cfg = binding.make_config(envs, agents, grid, 16, width=image[0], height=image[1])
    shape = binding.launch_shape(cfg, staged)
    assert shape.num_obs == envs * agents
    assert shape.tiles_x == -(-image[0] // 8) and shape.tiles_per_obs == shape.tiles_x * -(-image[1] // 8)
    assert 0 < shape.lds_bytes <= 160 * 1024 and shape.threads in (256, 512, 768, 1024)
    assert shape.obs_per_xcd * 8 >= shape.num_obs and 0 <= shape.obs_body_per_xcd <= shape.obs_per_xcd
    assert shape.tiles_per_block >= 1 and shape.blocks_per_obs * shape.tiles_per_block >= shape.tiles_per_obs
    assert (shape.blocks_per_obs - 1) * shape.tiles_per_block < shape.tiles_per_obs          # no empty strip
    assert shape.blocks_per_obs_tail * shape.tiles_per_block_tail >= shape.tiles_per_obs
    assert (shape.blocks_per_obs_tail - 1) * shape.tiles_per_block_tail < shape.tiles_per_obs
    covered = {}
    for obs, begin, end, _ in _work_list(shape):
        assert 0 <= begin < end <= shape.tiles_per_obs
        spans = covered.setdefault(obs, [])
        spans.append((begin, end))
    assert sorted(covered) == list(range(shape.num_obs))
    for obs, spans in covered.items():
        spans.sort()
        assert spans[0][0] == 0 and spans[-1][1] == shape.tiles_per_obs, obs
        assert all(a[1] == b[0] for a, b in zip(spans, spans[1:])), (obs, spans[:4])


def test_launch_shape_follows_the_staged_layers_and_rejects_what_create_rejects(lib):
    cfg = binding.make_config(4096, 2, (40, 40, 16), 16)
    full, low = binding.launch_shape(cfg, 0), binding.launch_shape(cfg, 10)
    assert low.lds_bytes < full.lds_bytes                 # fewer layers on chip, smaller workgroups' share
    assert full.lds_bytes - low.lds_bytes == 6 * 4 * 40 * 8      # four row arrays of 40 rows of 8 bytes per layer
    assert low.threads * (160 * 1024 // low.lds_bytes) >= 2048 or low.threads == 1024        # the CU's 32 wave slots are filled
    with pytest.raises(binding.MvError) as e:
        binding.launch_shape(cfg, 17)
    assert e.value.code == binding.MV_ERR_RANGE
    bad = binding.make_config(4, 1, (40, 40, 16), 16, width=0)
    with pytest.raises(binding.MvError) as e:
        binding.launch_shape(bad)
    assert e.value.code == binding.MV_ERR_ARG
    huge = binding.make_config(4, 1, (4096, 4096, 8), 16)
    with pytest.raises(binding.MvError) as e:
        binding.launch_shape(huge)
    assert e.value.code == binding.MV_ERR_CAPACITY
