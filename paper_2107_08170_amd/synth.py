"""Seeded synthetic voxel worlds and camera batches.

The paper's workloads are procedurally generated voxel scenarios (Sec. 4: worlds
with a floor, walls, elevated terrain, movable boxes, 1-4 agents, random
monochrome materials per episode; App. A.2: 128x72 observations).  Their
generators are not public inside the paper, so the five workloads below stand in
for them.  This module only draws random layouts and camera poses with NumPy; it
contains none of the renderer's arithmetic and is the only code that both the
HIP library's tests and the CPU oracle's tests consume.

Conventions: a world is ``u8[N, Z, Y, X]`` of material ids (0 = empty, x
fastest, z up, unit voxels); a palette is ``u8[N, M+1, 3]`` (row 0 unused); a
camera row is ``f32[x, y, z, yaw, pitch]`` with observation index
``env * A + agent``.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Iterator, Optional, Tuple

import numpy as np

BASE_SEED = 210708170


@dataclass(frozen=True)
class WorkloadSpec:
    """Static shape of one workload."""
    name: str
    index: int
    num_envs: int
    agents_per_env: int
    grid: Tuple[int, int, int]          # X, Y, Z
    width: int
    height: int
    num_materials: int
    steps: int                          # camera re-draws in the sustained loop
    dynamic: bool = False               # grids rewritten every step
    hfov_rad: float = float(np.float32(np.pi / 2))

    @property
    def num_obs(self) -> int:
        return self.num_envs * self.agents_per_env


SPECS = (
    WorkloadSpec("cfg0_tiny_4x1_16x16x8", 0, 4, 1, (16, 16, 8), 128, 72, 8, 1),
    WorkloadSpec("cfg1_256x4_40x40x16", 1, 256, 4, (40, 40, 16), 128, 72, 16, 1),
    WorkloadSpec("cfg2_4096x2_40x40x16_100steps", 2, 4096, 2, (40, 40, 16), 128, 72, 16, 100),
    WorkloadSpec("cfg3_1024x4_40x40x16_dynamic", 3, 1024, 4, (40, 40, 16), 128, 72, 16, 100, True),
    WorkloadSpec("cfg4_2048x4_64x64x32_256x144", 4, 2048, 4, (64, 64, 32), 256, 144, 16, 1),
)


@dataclass
class Workload:
    spec: WorkloadSpec
    voxels: np.ndarray                  # u8[N,Z,Y,X] (step-0 grid for dynamic worlds)
    palette: np.ndarray                 # u8[N,M+1,3]
    cameras: np.ndarray                 # f32[steps,N*A,5]
    self_voxel: Optional[np.ndarray] = None   # i32[steps,N*A] or None
    # dynamic worlds only
    static_voxels: Optional[np.ndarray] = None
    _dyn: dict = field(default_factory=dict)


def _rng(index: int, seed_offset: int = 0) -> np.random.Generator:
    return np.random.default_rng(BASE_SEED + index + seed_offset)


def _column_world(top: np.ndarray, Z: int) -> np.ndarray:
    """Occupancy ``bool[N,Z,Y,X]`` of columns solid for k < top[n,j,i]."""
    k = np.arange(Z, dtype=np.int32)[None, :, None, None]
    return k < top[:, None, :, :]


def _draw_materials(rng, occ: np.ndarray, M: int) -> np.ndarray:
    ids = rng.integers(1, M + 1, size=occ.shape, dtype=np.uint8)
    return np.where(occ, ids, np.uint8(0)).astype(np.uint8)


def _pick_cells(rng, free: np.ndarray, A: int) -> np.ndarray:
    """A distinct free (j,i) cells per env: ``free`` is bool[N,Y,X]; returns i32[N,A] flat j*X+i."""
    N = free.shape[0]
    score = rng.random(size=free.shape)
    score = np.where(free, score, -1.0).reshape(N, -1)
    order = np.argsort(-score, axis=1, kind="stable")[:, :A]
    picked = np.take_along_axis(score, order, axis=1)
    if (picked < 0).any():
        raise ValueError("an environment has fewer free cells than agents")
    return order.astype(np.int32)


def _draw_view_angles(rng, shape) -> Tuple[np.ndarray, np.ndarray]:
    yaw = rng.uniform(0.0, 2.0 * np.pi, size=shape)
    pitch = rng.uniform(-np.pi / 6.0, np.pi / 6.0, size=shape)
    return yaw, pitch


def _cameras_from_cells(cells: np.ndarray, X: int, zc: np.ndarray, yaw, pitch) -> np.ndarray:
    j, i = np.divmod(cells, X)
    cams = np.stack([i + 0.5, j + 0.5, zc, yaw, pitch], axis=-1)
    return cams.astype(np.float32)


def _walls_and_pillars(rng, N, X, Y, interior: np.ndarray):
    """Heights (voxels above the base) of cell walls and pillars; max where both fall."""
    wall = (rng.random(size=(N, Y, X)) < 0.08) & interior
    wall_h = rng.integers(1, 5, size=(N, Y, X), dtype=np.int32)
    pillar = (rng.random(size=(N, Y, X)) < 0.02) & interior
    pillar_h = rng.integers(2, 9, size=(N, Y, X), dtype=np.int32)
    return np.maximum(np.where(wall, wall_h, 0), np.where(pillar, pillar_h, 0))


def _gen_tiny(spec: WorkloadSpec, rng) -> Workload:
    N, A = spec.num_envs, spec.agents_per_env
    X, Y, Z = spec.grid
    M = spec.num_materials
    palette = rng.integers(0, 256, size=(N, M + 1, 3), dtype=np.uint8)
    above = np.zeros((N, Y, X), dtype=np.int32)
    for n in range(N):
        for _ in range(12):
            along_x = bool(rng.integers(0, 2))
            i0 = int(rng.integers(0, X))
            j0 = int(rng.integers(0, Y))
            length = int(rng.integers(3, 9))
            h = int(rng.integers(1, 5))
            if along_x:
                above[n, j0, i0:min(X, i0 + length)] = np.maximum(above[n, j0, i0:min(X, i0 + length)], h)
            else:
                above[n, j0:min(Y, j0 + length), i0] = np.maximum(above[n, j0:min(Y, j0 + length), i0], h)
    occ = _column_world(above + 1, Z)
    vox = _draw_materials(rng, occ, M)
    cells = _pick_cells(rng, above == 0, A)
    yaw, pitch = _draw_view_angles(rng, (spec.steps, N, A))
    zc = np.full((spec.steps, N, A), 1.5)
    cams = _cameras_from_cells(np.broadcast_to(cells, (spec.steps, N, A)), X, zc, yaw, pitch)
    return Workload(spec, vox, palette, cams.reshape(spec.steps, N * A, 5))


def _arena_heights(spec: WorkloadSpec, rng, N: int) -> np.ndarray:
    """Voxels above the floor for the 40x40 arena layout: perimeter 3, cell walls, pillars."""
    X, Y, _ = spec.grid
    border = np.zeros((Y, X), dtype=bool)
    border[0, :] = border[-1, :] = border[:, 0] = border[:, -1] = True
    above = _walls_and_pillars(rng, N, X, Y, ~border[None])
    return np.where(border[None], 3, above).astype(np.int32)


def _gen_arena(spec: WorkloadSpec, rng) -> Workload:
    N, A = spec.num_envs, spec.agents_per_env
    X, Y, Z = spec.grid
    M = spec.num_materials
    palette = rng.integers(0, 256, size=(N, M + 1, 3), dtype=np.uint8)
    above = _arena_heights(spec, rng, N)
    vox = _draw_materials(rng, _column_world(above + 1, Z), M)
    wl = Workload(spec, vox, palette, np.zeros((0, N * A, 5), np.float32))
    if spec.dynamic:
        _init_dynamic(wl, rng, above)
        return wl
    cells = _pick_cells(rng, above == 0, A)
    yaw, pitch = _draw_view_angles(rng, (spec.steps, N, A))
    zc = np.full((spec.steps, N, A), 1.5)
    cams = _cameras_from_cells(np.broadcast_to(cells, (spec.steps, N, A)), X, zc, yaw, pitch)
    wl.cameras = cams.reshape(spec.steps, N * A, 5)
    return wl


def _gen_terrain(spec: WorkloadSpec, rng) -> Workload:
    N, A = spec.num_envs, spec.agents_per_env
    X, Y, Z = spec.grid
    M = spec.num_materials
    palette = rng.integers(0, 256, size=(N, M + 1, 3), dtype=np.uint8)
    coarse = rng.integers(0, 7, size=(N, Y // 4, X // 4), dtype=np.int32)
    terrain = np.repeat(np.repeat(coarse, 4, axis=1), 4, axis=2)      # h: voxels k=0..h solid
    above = _walls_and_pillars(rng, N, X, Y, np.ones((1, Y, X), dtype=bool))
    vox = _draw_materials(rng, _column_world(terrain + 1 + above, Z), M)
    cells = _pick_cells(rng, above == 0, A)
    yaw, pitch = _draw_view_angles(rng, (spec.steps, N, A))
    h_at = np.take_along_axis(terrain.reshape(N, -1), cells, axis=1)
    zc = np.broadcast_to(h_at + 1.5, (spec.steps, N, A))
    cams = _cameras_from_cells(np.broadcast_to(cells, (spec.steps, N, A)), X, zc, yaw, pitch)
    return Workload(spec, vox, palette, cams.reshape(spec.steps, N * A, 5))


# ---------------------------------------------------------------- dynamic worlds (boxes + bodies)
NUM_BOXES = 32
_DIRS = np.array([[1, 0], [-1, 0], [0, 1], [0, -1]], dtype=np.int32)   # (di, dj)


def _init_dynamic(wl: Workload, rng, above: np.ndarray) -> None:
    spec = wl.spec
    N, A = spec.num_envs, spec.agents_per_env
    X, Y, Z = spec.grid
    M = spec.num_materials
    wl.static_voxels = wl.voxels
    cells = _pick_cells(rng, above == 0, NUM_BOXES + A)
    box_cells, agent_cells = cells[:, :NUM_BOXES].copy(), cells[:, NUM_BOXES:].copy()
    box_mat = rng.integers(1, M + 1, size=(N, NUM_BOXES), dtype=np.uint8)
    body_mat = rng.integers(1, M + 1, size=(N, A, 2), dtype=np.uint8)
    yaw, pitch = _draw_view_angles(rng, (N, A))
    wl._dyn = dict(rng=rng, box=box_cells, agent=agent_cells, box_mat=box_mat,
                   body_mat=body_mat, yaw=yaw, pitch=pitch, step=0)
    wl.voxels = dynamic_grid(wl)
    cams, selfv = dynamic_cameras(wl)
    wl.cameras, wl.self_voxel = cams[None], selfv[None]


def dynamic_grid(wl: Workload) -> np.ndarray:
    """Static arena with the movable boxes (1x1x1 at k=1) and agent bodies (1x1x2 at k=1..2) stamped in."""
    X, Y, _ = wl.spec.grid
    d = wl._dyn
    vox = wl.static_voxels.copy()
    n_idx = np.arange(vox.shape[0])[:, None]
    bj, bi = np.divmod(d["box"], X)
    vox[n_idx, 1, bj, bi] = d["box_mat"]
    aj, ai = np.divmod(d["agent"], X)
    vox[n_idx, 1, aj, ai] = d["body_mat"][:, :, 0]
    vox[n_idx, 2, aj, ai] = d["body_mat"][:, :, 1]
    return vox


def dynamic_cameras(wl: Workload) -> Tuple[np.ndarray, np.ndarray]:
    X, Y, _ = wl.spec.grid
    d = wl._dyn
    N, A = d["agent"].shape
    cams = _cameras_from_cells(d["agent"], X, np.full((N, A), 1.5), d["yaw"], d["pitch"])
    selfv = (1 * Y * X + d["agent"]).astype(np.int32)      # lower body voxel (i,j,1)
    return cams.reshape(N * A, 5), selfv.reshape(N * A)


def dynamic_step(wl: Workload) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Advance the toy dynamics one step: agents, then boxes, in index order, each moving one
    cell along +-x/+-y unless the target is solid or on the perimeter; view angles re-drawn.
    Returns (voxels, cameras, self_voxel) of the new step."""
    spec = wl.spec
    X, Y, _ = spec.grid
    d = wl._dyn
    rng = d["rng"]
    N, A = d["agent"].shape
    n_idx = np.arange(N)
    cur = dynamic_grid(wl)
    adir = rng.integers(0, 4, size=(N, A))
    bdir = rng.integers(0, 4, size=(N, NUM_BOXES))

    def try_move(cells_col, dirs, tall, mats):
        j, i = np.divmod(cells_col, X)
        ti, tj = i + _DIRS[dirs, 0], j + _DIRS[dirs, 1]
        inside = (ti >= 1) & (ti <= X - 2) & (tj >= 1) & (tj <= Y - 2)
        tic, tjc = np.clip(ti, 0, X - 1), np.clip(tj, 0, Y - 1)
        free = cur[n_idx, 1, tjc, tic] == 0
        if tall:
            free &= cur[n_idx, 2, tjc, tic] == 0
        ok = inside & free
        # vacate, then occupy
        m_lo = cur[n_idx, 1, j, i].copy()
        cur[n_idx[ok], 1, j[ok], i[ok]] = 0
        cur[n_idx[ok], 1, tj[ok], ti[ok]] = m_lo[ok]
        if tall:
            m_hi = cur[n_idx, 2, j, i].copy()
            cur[n_idx[ok], 2, j[ok], i[ok]] = 0
            cur[n_idx[ok], 2, tj[ok], ti[ok]] = m_hi[ok]
        return np.where(ok, tj * X + ti, cells_col).astype(np.int32)

    for a in range(A):
        d["agent"][:, a] = try_move(d["agent"][:, a], adir[:, a], True, None)
    for b in range(NUM_BOXES):
        d["box"][:, b] = try_move(d["box"][:, b], bdir[:, b], False, None)
    d["yaw"], d["pitch"] = _draw_view_angles(rng, (N, A))
    d["step"] += 1
    cams, selfv = dynamic_cameras(wl)
    return cur, cams, selfv


def dynamic_positions(wl: Workload) -> Tuple[np.ndarray, np.ndarray]:
    """Copies of the current floor cells (j*X+i) of the boxes i32[N,32] and of the agents i32[N,A]."""
    return wl._dyn["box"].copy(), wl._dyn["agent"].copy()


def object_moves(wl: Workload, before: Tuple[np.ndarray, np.ndarray],
                 after: Tuple[np.ndarray, np.ndarray]) -> Tuple[np.ndarray, np.ndarray, np.ndarray, np.ndarray]:
    """The step from ``before`` to ``after`` (two results of dynamic_positions) as one entry per object voxel:
    (env i32[n], from_voxel i32[n], to_voxel i32[n], material u8[n]); boxes are one voxel at k=1, agent bodies two
    (k=1 and k=2).  Objects that stayed where they were are listed too (from == to)."""
    X, Y, _ = wl.spec.grid
    d = wl._dyn
    N = before[0].shape[0]
    plane = X * Y
    env, frm, to, mat = [], [], [], []

    def add(cells_before, cells_after, layer, materials):
        n_idx = np.broadcast_to(np.arange(N, dtype=np.int32)[:, None], cells_before.shape)
        env.append(n_idx.reshape(-1)); frm.append((layer * plane + cells_before).reshape(-1))
        to.append((layer * plane + cells_after).reshape(-1)); mat.append(materials.reshape(-1))

    add(before[0], after[0], 1, d["box_mat"])
    add(before[1], after[1], 1, d["body_mat"][:, :, 0])
    add(before[1], after[1], 2, d["body_mat"][:, :, 1])
    return (np.concatenate(env).astype(np.int32), np.concatenate(frm).astype(np.int32),
            np.concatenate(to).astype(np.int32), np.concatenate(mat).astype(np.uint8))


def grid_edits(before: np.ndarray, after: np.ndarray) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """The voxels that differ between two batches of grids, as (env i32[n], voxel_index i32[n],
    material u8[n]) with the material of ``after``: each changed voxel appears exactly once."""
    N = before.shape[0]
    diff = np.nonzero(before.reshape(N, -1) != after.reshape(N, -1))
    env = diff[0].astype(np.int32)
    idx = diff[1].astype(np.int32)
    return env, idx, after.reshape(N, -1)[diff].astype(np.uint8)


def generate(index: int, num_envs: Optional[int] = None, steps: Optional[int] = None,
             seed_offset: int = 0) -> Workload:
    """Build workload ``index`` (0-4).  ``num_envs``/``steps`` shrink it for bounded samples;
    the layout of the first environments does not depend on ``steps`` but does depend on
    ``num_envs`` (draws are vectorised over environments)."""
    spec = SPECS[index]
    if num_envs is not None or steps is not None:
        spec = WorkloadSpec(spec.name, spec.index, num_envs or spec.num_envs, spec.agents_per_env,
                            spec.grid, spec.width, spec.height, spec.num_materials,
                            steps or spec.steps, spec.dynamic, spec.hfov_rad)
    rng = _rng(index, seed_offset)
    if index == 0:
        return _gen_tiny(spec, rng)
    if index == 4:
        return _gen_terrain(spec, rng)
    return _gen_arena(spec, rng)


# Workloads for the render paths the five headline workloads never take (same arena recipe, mid-size batches):
#   wide    : grids wider than 64 voxels (rows of more than one word): the per-cell tracer over rows staged on chip
#   outside : cameras outside the grid, looking in: the per-cell tracer over rows in device memory
#   odd     : an image whose width and height are not multiples of the 8x8 tile: clamped tiles and byte stores
EXTRA_SPECS = {
    "wide": WorkloadSpec("wide_256x2_96x96x16", 5, 256, 2, (96, 96, 16), 128, 72, 16, 1),
    "outside": WorkloadSpec("outside_256x4_40x40x16", 6, 256, 4, (40, 40, 16), 128, 72, 16, 1),
    "odd": WorkloadSpec("odd_256x4_40x40x16_130x70", 7, 256, 4, (40, 40, 16), 130, 70, 16, 1),
}


def generate_extra(name: str) -> Workload:
    """One of the EXTRA_SPECS workloads (seed = BASE_SEED + its index)."""
    spec = EXTRA_SPECS[name]
    rng = _rng(spec.index)
    wl = _gen_arena(spec, rng)
    if name == "outside":
        # every camera on a ring around its arena, above the walls, looking at the middle (give or take)
        N, A = spec.num_envs, spec.agents_per_env
        X, Y, Z = spec.grid
        n = N * A
        around = rng.uniform(0.0, 2.0 * np.pi, size=n)
        radius = rng.uniform(0.6 * X, 0.95 * X, size=n)
        pos = np.stack([X / 2 + radius * np.cos(around), Y / 2 + radius * np.sin(around),
                        rng.uniform(2.0, Z - 2.0, size=n)], axis=1)
        yaw = around + np.pi + rng.uniform(-0.3, 0.3, size=n)
        pitch = rng.uniform(-0.45, 0.05, size=n)
        wl.cameras = np.concatenate([pos, yaw[:, None], pitch[:, None]], axis=1).astype(np.float32)[None]
    return wl


def random_world(rng: np.random.Generator, N: int, grid: Tuple[int, int, int], fill: float,
                 M: int) -> Tuple[np.ndarray, np.ndarray]:
    """Unstructured worlds (i.i.d. occupancy with probability ``fill``) for edge-case tests:
    overhangs, floating voxels, no floor."""
    X, Y, Z = grid
    occ = rng.random(size=(N, Z, Y, X)) < fill
    vox = _draw_materials(rng, occ, M)
    palette = rng.integers(0, 256, size=(N, M + 1, 3), dtype=np.uint8)
    return vox, palette


def random_cameras(rng: np.random.Generator, count: int, grid: Tuple[int, int, int],
                   margin: float = 0.0, max_pitch: float = np.pi / 2) -> np.ndarray:
    """Cameras at uniformly random continuous positions in the grid box grown by ``margin``
    voxels on each side (so some start outside when margin > 0), any yaw, pitch in +-max_pitch."""
    X, Y, Z = grid
    lo = np.array([-margin] * 3)
    hi = np.array([X + margin, Y + margin, Z + margin])
    pos = rng.uniform(lo, hi, size=(count, 3))
    yaw = rng.uniform(0.0, 2.0 * np.pi, size=(count, 1))
    pitch = rng.uniform(-max_pitch, max_pitch, size=(count, 1))
    return np.concatenate([pos, yaw, pitch], axis=1).astype(np.float32)
