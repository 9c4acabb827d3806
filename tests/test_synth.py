"""The seeded input generators: same seed => same arrays, and the worlds have the structure the design
document states (floor, perimeter, empty camera cells, distinct agent cells, material range, toy
dynamics that conserve boxes and bodies).  CPU only; no renderer arithmetic is involved."""
import hashlib

import numpy as np
import pytest

from paper_2107_08170_amd import synth


def _digest(wl) -> str:
    h = hashlib.sha256()
    for a in (wl.voxels, wl.palette, wl.cameras):
        h.update(np.ascontiguousarray(a).tobytes())
    if wl.self_voxel is not None:
        h.update(np.ascontiguousarray(wl.self_voxel).tobytes())
    return h.hexdigest()


@pytest.mark.parametrize("index,envs", [(0, None), (1, 16), (2, 16), (3, 16), (4, 4)])
def test_same_seed_same_arrays(index, envs):
    a = synth.generate(index, num_envs=envs)
    b = synth.generate(index, num_envs=envs)
    assert _digest(a) == _digest(b)
    c = synth.generate(index, num_envs=envs, seed_offset=1)
    assert _digest(a) != _digest(c)


@pytest.mark.parametrize("index,envs", [(0, None), (1, 32), (2, 32), (3, 32), (4, 8)])
def test_shapes_types_and_material_range(index, envs):
    wl = synth.generate(index, num_envs=envs, steps=3 if index == 2 else None)
    s = wl.spec
    X, Y, Z = s.grid
    assert wl.voxels.shape == (s.num_envs, Z, Y, X) and wl.voxels.dtype == np.uint8
    assert wl.palette.shape == (s.num_envs, s.num_materials + 1, 3) and wl.palette.dtype == np.uint8
    assert wl.cameras.dtype == np.float32 and wl.cameras.shape[1:] == (s.num_obs, 5)
    assert int(wl.voxels.max()) <= s.num_materials
    assert (wl.voxels[:, 0] != 0).all(), "the floor layer is solid everywhere"
    # every material id is in use somewhere (i.i.d. uniform draw over thousands of solid voxels)
    assert set(np.unique(wl.voxels)) >= set(range(1, s.num_materials + 1))


@pytest.mark.parametrize("index", [1, 2, 3])
def test_arena_structure(index):
    wl = synth.generate(index, num_envs=24, steps=2 if index == 2 else None)
    s = wl.spec
    X, Y, Z = s.grid
    occ = wl.voxels != 0
    # perimeter walls: exactly three voxels above the floor
    edge = np.zeros((Y, X), bool)
    edge[0, :] = edge[-1, :] = edge[:, 0] = edge[:, -1] = True
    assert occ[:, 1:4][:, :, edge].all() and not occ[:, 4:][:, :, edge].any()
    # columns: solid from the floor up without gaps, except the stamped bodies/boxes of the dynamic world
    static = (wl.static_voxels if s.dynamic else wl.voxels) != 0
    heights = static.sum(axis=1)
    assert (static == (np.arange(Z)[None, :, None, None] < heights[:, None])).all()
    assert heights.max() <= 9
    # cameras: centre of a cell that is empty in the static world, eye at 1.5, pitch within +-30 degrees
    cams = wl.cameras[0].reshape(s.num_envs, s.agents_per_env, 5)
    i = np.floor(cams[..., 0]).astype(int); j = np.floor(cams[..., 1]).astype(int)
    assert np.allclose(cams[..., 0] - i, 0.5) and np.allclose(cams[..., 1] - j, 0.5) and np.allclose(cams[..., 2], 1.5)
    n = np.arange(s.num_envs)[:, None]
    assert (heights[n, j, i] == 1).all(), "camera cells carry nothing but the floor"
    assert (np.abs(cams[..., 4]) <= np.pi / 6 + 1e-6).all() and (cams[..., 3] >= 0).all() and (cams[..., 3] < 2 * np.pi + 1e-6).all()
    # agents of one environment stand in distinct cells
    cell = j * X + i
    assert all(len(set(row)) == s.agents_per_env for row in cell)


def test_tiny_and_terrain_camera_cells():
    for index, envs in ((0, None), (4, 8)):
        wl = synth.generate(index, num_envs=envs)
        s = wl.spec
        X, Y, Z = s.grid
        occ = wl.voxels != 0
        heights = occ.sum(axis=1)
        cams = wl.cameras[0].reshape(s.num_envs, s.agents_per_env, 5)
        i = np.floor(cams[..., 0]).astype(int); j = np.floor(cams[..., 1]).astype(int)
        n = np.arange(s.num_envs)[:, None]
        top = heights[n, j, i]
        assert np.allclose(cams[..., 2], top + 0.5), "eye half a voxel above the top of its column"
        k = np.floor(cams[..., 2]).astype(int)
        assert not occ[n, k, j, i].any(), "the camera's own voxel is empty"


def test_dynamic_world_conserves_boxes_and_bodies_and_edits_replay():
    wl = synth.generate(3, num_envs=12)
    s = wl.spec
    X, Y, Z = s.grid
    N, A = s.num_envs, s.agents_per_env
    static = wl.static_voxels != 0
    grid = wl.voxels
    cams, selfv = wl.cameras[0], wl.self_voxel[0]
    for _ in range(4):
        movable = (grid != 0) & ~static
        assert (movable.reshape(N, -1).sum(axis=1) == synth.NUM_BOXES + 2 * A).all()
        assert not movable[:, 0].any() and not movable[:, 3:].any(), "boxes and bodies live in layers 1 and 2"
        # the self voxel of every camera is the lower voxel of a two-voxel body in the camera's own cell
        k, rem = np.divmod(selfv, X * Y); j, i = np.divmod(rem, X)
        env = np.repeat(np.arange(N), A)
        assert (k == 1).all() and (grid[env, 1, j, i] != 0).all() and (grid[env, 2, j, i] != 0).all()
        assert (np.floor(cams[:, 0]) == i).all() and (np.floor(cams[:, 1]) == j).all()
        before = grid
        grid, cams, selfv = synth.dynamic_step(wl)
        e, idx, mat = synth.grid_edits(before, grid)
        assert len(np.unique(e.astype(np.int64) * before[0].size + idx)) == e.size, "each changed voxel appears once"
        replay = before.copy().reshape(N, -1)
        replay[e, idx] = mat
        assert (replay.reshape(grid.shape) == grid).all()
        assert e.size > 0
