"""Pins for the CPU oracle (CPU only).  Each test fixes the oracle to something other than itself:
brute-force definition D, closed forms of the pinhole geometry, invariances, exact rational
rounding.  A dropped term, wrong sign, swapped axis or transposed index in oracle/mv_oracle.c
fails at least one of them."""
import os
from fractions import Fraction

import numpy as np
import pytest

from paper_2107_08170_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
W, H = 128, 72
HFOV = float(np.float32(np.pi / 2))


def _read_table(name):
    rows = []
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            rows.append([float(x) for x in line.split()])
    return rows


def _single(orc, grid, vox, palette, cams, self_voxel=None, w=W, h=H, **kw):
    """Oracle render of one environment with len(cams) agents."""
    cams = np.asarray(cams, np.float32).reshape(-1, 5)
    M = palette.shape[0] - 1
    b = orc.OracleBatch(1, cams.shape[0], grid, w, h, M, **kw)
    b.upload_worlds(vox[None], palette[None])
    b.set_cameras(cams, self_voxel)
    return b, b.render()


# --------------------------------------------------------------------------- P1: brute force
@pytest.mark.parametrize("seed", range(6))
def test_dda_matches_definition_on_tiny_grids(orc, seed):
    """Algorithm O == definition D (every solid voxel slab-tested) on grids <= 8x8x4, random
    occupancy 0-50 %, cameras inside, outside and inside solids, with and without own body."""
    rng = np.random.default_rng(1000 + seed)
    w, h = 32, 18
    checked = 0
    for trial in range(8):
        grid = (int(rng.integers(1, 9)), int(rng.integers(1, 9)), int(rng.integers(1, 5)))
        fill = float(rng.uniform(0.0, 0.5))
        vox, pal = synth.random_world(rng, 1, grid, fill, 5)
        cams = synth.random_cameras(rng, 3, grid, margin=2.0)
        X, Y, Z = grid
        selfv = np.full(3, -1, np.int32)
        if trial % 2:       # give camera 0 a body at the voxel it stands in (if inside the grid)
            c = np.floor(cams[0, :3]).astype(int)
            if (c >= 0).all() and c[0] < X and c[1] < Y and c[2] < Z:
                selfv[0] = (c[2] * Y + c[1]) * X + c[0]
        b, out = _single(orc, grid, vox[0], pal[0], cams, selfv, w=w, h=h)
        for a in range(3):
            rays = b.pixel_rays(a).reshape(-1, 3).astype(np.float64)
            P = np.broadcast_to(b.camera_record(a)[:3].astype(np.float64), rays.shape)
            hit, face, t = orc.definition_first_hit(grid, vox[0], P, rays,
                                                    np.full(rays.shape[0], selfv[a], np.int32))
            ok = out.edge_margin[a].reshape(-1) > 1e-9
            assert ok.mean() > 0.99
            np.testing.assert_array_equal(out.hit_index[a].reshape(-1)[ok], hit[ok])
            o_face = out.face[a].reshape(-1).astype(np.int32)
            np.testing.assert_array_equal(o_face[ok], face[ok])
            np.testing.assert_allclose(out.t[a].reshape(-1)[ok], t[ok], rtol=0, atol=1e-12)
            checked += int(ok.sum())
    assert checked > 10000


def test_definition_on_structured_world(orc):
    """Same comparison on the tiny workload's real layout (floor, walls), full resolution rows."""
    wl = synth.generate(0)
    s = wl.spec
    b = orc.OracleBatch(s.num_envs, s.agents_per_env, s.grid, s.width, s.height, s.num_materials)
    b.upload_worlds(wl.voxels, wl.palette)
    b.set_cameras(wl.cameras[0])
    out = b.render()
    for o in range(s.num_obs):
        rays = b.pixel_rays(o)[::4, ::4].reshape(-1, 3).astype(np.float64)
        P = np.broadcast_to(b.camera_record(o)[:3].astype(np.float64), rays.shape)
        hit, face, t = orc.definition_first_hit(s.grid, wl.voxels[o], P, rays)
        ok = out.edge_margin[o][::4, ::4].reshape(-1) > 1e-9
        np.testing.assert_array_equal(out.hit_index[o][::4, ::4].reshape(-1)[ok], hit[ok])
        np.testing.assert_array_equal(out.face[o][::4, ::4].reshape(-1)[ok].astype(np.int32), face[ok])
        np.testing.assert_allclose(out.t[o][::4, ::4].reshape(-1)[ok], t[ok], atol=1e-12, rtol=0)


# --------------------------------------------------------------------------- P2: single cube
def _cube_case(orc, yaw, pitch, D, axis_dir):
    """Camera at the centre of a 17^3 grid looking along axis_dir (unit int vector); one solid voxel
    on the optical axis whose near face is at planar distance D."""
    grid = (34, 34, 34)
    cam_cell = np.array([17, 17, 17])
    vox = np.zeros((34, 34, 34), np.uint8)
    cube = cam_cell + np.array(axis_dir) * D
    vox[cube[2], cube[1], cube[0]] = 3
    pal = np.zeros((6, 3), np.uint8)
    pal[3] = (200, 100, 51)
    # camera sits on the boundary plane of its cell along the view axis so that the near-face distance
    # is exactly D: position = cell centre shifted by half a voxel backwards along axis_dir.
    pos = cam_cell + 0.5 - 0.5 * np.array(axis_dir) + (np.array(axis_dir) < 0) * 0.0
    # near face plane coordinate along the axis: cube (if dir>0) or cube+1 (if dir<0)
    a = int(np.argmax(np.abs(axis_dir)))
    near = cube[a] if axis_dir[a] > 0 else cube[a] + 1
    pos[a] = near - axis_dir[a] * D
    cam = [pos[0], pos[1], pos[2], yaw, pitch]
    _, out = _single(orc, grid, vox, pal, [cam])
    return out, (cube[2] * 34 + cube[1]) * 34 + cube[0]


@pytest.mark.parametrize("D,c0,c1,r0,r1,count,depth", _read_table("single_cube_footprint.txt"))
def test_single_cube_footprint_and_depth(orc, D, c0, c1, r0, r1, count, depth):
    D, c0, c1, r0, r1, count = int(D), int(c0), int(c1), int(r0), int(r1), int(count)
    out, cube_idx = _cube_case(orc, 0.0, 0.0, D, (1, 0, 0))
    hit = out.hit_index[0] >= 0
    assert hit.sum() == count
    rows, cols = np.nonzero(hit)
    assert (rows.min(), rows.max(), cols.min(), cols.max()) == (r0, r1, c0, c1)
    assert hit[r0:r1 + 1, c0:c1 + 1].all()
    assert (out.hit_index[0][hit] == cube_idx).all()
    assert (out.face[0][hit] == 0).all()                      # entered through the -x face
    assert (out.depth[0][hit] == np.float32(depth)).all()     # planar depth, exactly D
    assert (out.depth[0][~hit] == 0).all()
    # colour: palette * 0.30 (the -x face is unlit by the default light), rounded to nearest
    expected = [int(Fraction(v) * Fraction(float(np.float32(0.3))) + Fraction(1, 2)) for v in (200, 100, 51)]
    assert (out.rgb[0][hit] == np.array(expected, np.uint8)).all()
    assert (out.rgb[0][~hit] == np.array((135, 206, 235), np.uint8)).all()


_FACE_CASES = [
    # yaw, pitch, view direction, face entered
    (0.0, 0.0, (1, 0, 0), 0),
    (np.pi, 0.0, (-1, 0, 0), 1),
    (np.pi / 2, 0.0, (0, 1, 0), 2),
    (-np.pi / 2, 0.0, (0, -1, 0), 3),
    (0.3, np.pi / 2, (0, 0, 1), 4),
    (1.1, -np.pi / 2, (0, 0, -1), 5),
]


@pytest.mark.parametrize("yaw,pitch,direction,face", _FACE_CASES)
def test_six_faces_and_intensities(orc, yaw, pitch, direction, face):
    """Looking along each of the six axis directions pins yaw/pitch sign conventions, the face
    numbering and the Lambert table (golden: ambient + diffuse*max(0,n.L))."""
    golden = {int(r[0]): r[1] for r in _read_table("face_intensity_default.txt")}
    out, cube_idx = _cube_case(orc, yaw, pitch, 4, direction)
    hit = out.hit_index[0] >= 0
    # yaw/pitch are float32-rounded, so the footprint edge may move by a pixel row/col; the core must hit
    assert hit[30:42, 58:70].all()
    assert 200 <= hit.sum() <= 320
    assert (out.hit_index[0][hit] == cube_idx).all()
    core = np.zeros_like(hit)
    core[30:42, 58:70] = True
    assert (out.face[0][core] == face).all()
    np.testing.assert_allclose(out.depth[0][core], 4.0, rtol=1e-6)
    I = golden[face]
    for ch, v in enumerate((200, 100, 51)):
        exact = v * I + 0.5
        got = out.rgb[0][core][:, ch]
        assert (np.abs(got.astype(int) - int(exact)) <= (1 if abs(exact - round(exact)) < 1e-3 else 0)).all()


def test_face_intensity_table(orc):
    golden = [r[1] for r in _read_table("face_intensity_default.txt")]
    b = orc.OracleBatch(1, 1, (2, 2, 2), 8, 8, 1)
    np.testing.assert_allclose(b.face_intensity(), np.array(golden, np.float32), rtol=0, atol=6e-8)
    # a different light: only the lit faces change, each by its own component
    b2 = orc.OracleBatch(1, 1, (2, 2, 2), 8, 8, 1, light_dir=(-2.0, 0.0, -1.0), ambient=0.1, diffuse=0.5)
    s5 = np.sqrt(5.0)
    np.testing.assert_allclose(b2.face_intensity(),
                               [0.1 + 0.5 * 2 / s5, 0.1, 0.1, 0.1, 0.1 + 0.5 / s5, 0.1, 0.1], atol=1e-7)


def test_off_axis_cube_pins_left_right_and_up_down(orc):
    """A voxel to the LEFT of and ABOVE the optical axis must appear at small column and small row
    indices: with yaw 0 the camera looks along +x, its right is -y, its up is +z."""
    grid = (16, 16, 16)
    vox = np.zeros((16, 16, 16), np.uint8)
    vox[10, 10, 8] = 1                           # voxel i=8, j=10, k=10
    pal = np.full((2, 3), 255, np.uint8)
    cam = [2.0, 8.5, 8.5, 0.0, 0.0]              # near face x=8 at planar distance 6
    _, out = _single(orc, grid, vox, pal, [cam])
    front = out.face[0] == 0
    # closed form: ray reaches the plane x=8 at y = 8.5 - 6*sx, z = 8.5 + 6*sy*(72/128)
    c = np.arange(W)
    r = np.arange(H)
    y = 8.5 - 6.0 * (2 * c + 1 - W) / W
    z = 8.5 + 6.0 * (H - 2 * r - 1) / H * (H / W)
    expect = ((z > 10) & (z < 11))[:, None] & ((y > 10) & (y < 11))[None, :]
    assert expect.sum() > 100
    np.testing.assert_array_equal(front, expect)
    rows, cols = np.nonzero(front)
    assert cols.max() < W // 2 and rows.max() < H // 2      # left of and above the image centre
    np.testing.assert_array_equal(out.depth[0][front], np.float32(6.0))
    # the -y and -z side faces of the voxel face the camera too and are seen beyond the front face
    assert (out.face[0] == 2).any() and (out.face[0] == 4).any()
    assert not (out.face[0] == 3).any() and not (out.face[0] == 5).any() and not (out.face[0] == 1).any()


# --------------------------------------------------------------------------- P3: floor depth
def test_floor_depth_closed_form(orc):
    table = {int(r[0]): r[1] for r in _read_table("floor_depth_rows.txt")}
    grid = (40, 40, 4)
    vox = np.zeros((4, 40, 40), np.uint8)
    vox[0] = 2
    pal = np.array([[0, 0, 0], [9, 9, 9], [100, 150, 250]], np.uint8)
    cam = [20.5, 20.5, 1.5, 0.7, 0.0]
    b, out = _single(orc, grid, vox, pal, [cam])
    assert (out.hit_index[0][:H // 2] == -1).all()           # above the horizon: sky
    rec = b.camera_record(0).astype(np.float64)
    rays = b.pixel_rays(0).astype(np.float64)
    for r in range(H // 2, H):
        depth = table[r]
        pts = rec[:3] + depth * rays[r]                      # where the closed form says the ray lands
        inside = (pts[:, 0] > 0) & (pts[:, 0] < 40) & (pts[:, 1] > 0) & (pts[:, 1] < 40)
        row = out.depth[0][r]
        np.testing.assert_allclose(row[inside], depth, rtol=2e-7)
        assert (out.face[0][r][inside] == 5).all()           # top (+z) face of the floor
        assert (out.hit_index[0][r][inside] < 1600).all()
        assert (row[~inside] == 0).all()                     # floor point beyond the grid: miss
        # hit voxel is the floor cell under the landing point
        ij = np.floor(pts[inside][:, :2]).astype(int)
        margin = np.abs(pts[inside][:, :2] - np.round(pts[inside][:, :2])).min(axis=1)
        sel = margin > 1e-6
        np.testing.assert_array_equal(out.hit_index[0][r][inside][sel], (ij[:, 1] * 40 + ij[:, 0])[sel])
    assert inside.any()
    # colour: lit top face, I = 0.3 + 0.7*3/sqrt(14)
    I = float(np.float32(0.3 + 0.7 * 3 / np.sqrt(14.0)))
    exp = [int(Fraction(v) * Fraction(I) + Fraction(1, 2)) for v in (100, 150, 250)]
    assert (out.rgb[0][H - 1][out.hit_index[0][H - 1] >= 0] == np.array(exp, np.uint8)).all()


# --------------------------------------------------------------------------- P4: empty world
def test_empty_world_is_sky(orc):
    grid = (7, 5, 3)
    vox = np.zeros((3, 5, 7), np.uint8)
    pal = np.full((3, 3), 77, np.uint8)
    rng = np.random.default_rng(5)
    cams = synth.random_cameras(rng, 4, grid, margin=3.0)
    _, out = _single(orc, grid, vox, pal, cams, sky_rgb=(1, 2, 3))
    assert (out.rgb == np.array((1, 2, 3), np.uint8)).all()
    assert (out.depth == 0).all() and (out.depth.view(np.uint32) == 0).all()
    assert (out.hit_index == -1).all() and (out.material == 0).all() and (out.face == 255).all()


# --------------------------------------------------------------------------- P5: invariances
def _render_world(orc, grid, vox, pal, cams, **kw):
    _, out = _single(orc, grid, vox, pal, cams, **kw)
    return out


def _arena(seed, grid=(12, 9, 6)):
    rng = np.random.default_rng(seed)
    vox, pal = synth.random_world(rng, 1, grid, 0.12, 7)
    vox[0, 0] = rng.integers(1, 8, size=vox[0, 0].shape, dtype=np.uint8)     # a floor
    return rng, vox[0], pal[0]


def test_rotation_by_90_degrees_about_z(orc):
    """Rotate grid and camera together: (i,j,k)->(Y-1-j,i,k), (x,y,psi)->(Y-y,x,psi+pi/2).
    Depth and material images are unchanged; hit indices map through the permutation; colours are
    unchanged when the light is rotated too, and follow the face permutation when it is not."""
    X, Y, Z = 12, 9, 6
    rng, vox, pal = _arena(11, (X, Y, Z))
    # exactly representable poses so that the rotated camera is the same camera, bit for bit, up to
    # the float32 rounding of yaw+pi/2 (hence the small tolerances below)
    cams = np.array([[3.5, 4.5, 1.5, 0.25, 0.125], [7.25, 2.75, 2.5, 2.0, -0.375]], np.float32)
    rot = np.zeros((Z, X, Y), np.uint8)             # new dims (X'=Y, Y'=X)
    for j in range(Y):
        for i in range(X):
            rot[:, i, Y - 1 - j] = vox[:, j, i]
    cams_r = cams.copy()
    cams_r[:, 0] = Y - cams[:, 1]
    cams_r[:, 1] = cams[:, 0]
    cams_r[:, 3] = cams[:, 3] + np.float32(np.pi / 2)
    light = (1.0, 2.0, 3.0)
    light_r = (-2.0, 1.0, 3.0)                      # (lx,ly) -> (-ly,lx)
    a = _render_world(orc, (X, Y, Z), vox, pal, cams, light_dir=light)
    b = _render_world(orc, (Y, X, Z), rot, pal, cams_r, light_dir=light_r)
    ok = (a.edge_margin > 1e-5) & (b.edge_margin > 1e-5)
    assert ok.mean() > 0.97
    np.testing.assert_array_equal(a.material[ok], b.material[ok])
    # float32(yaw + pi/2) is not the exactly rotated yaw: grazing rays move by a few 1e-6 relative
    np.testing.assert_allclose(a.depth[ok], b.depth[ok], rtol=2e-5)
    hit = ok & (a.hit_index >= 0)
    k, rem = np.divmod(a.hit_index[hit], X * Y)
    j, i = np.divmod(rem, X)
    np.testing.assert_array_equal(b.hit_index[hit], (k * X + i) * Y + (Y - 1 - j))
    np.testing.assert_array_equal((a.hit_index < 0)[ok], (b.hit_index < 0)[ok])
    np.testing.assert_array_equal(a.rgb[ok], b.rgb[ok])
    # faces permute: -x->-y? outward normal (nx,ny)->(-ny,nx): -x(0)->-y(2), +x(1)->+y(3), -y(2)->+x(1), +y(3)->-x(0)
    perm = np.array([2, 3, 1, 0, 4, 5, 6], np.uint8)
    np.testing.assert_array_equal(perm[a.face[hit]], b.face[hit])
    # light NOT rotated: colours differ exactly as the permuted faces predict
    c = _render_world(orc, (Y, X, Z), rot, pal, cams_r, light_dir=light)
    I = orc.OracleBatch(1, 1, (2, 2, 2), 8, 8, 1, light_dir=light).face_intensity()
    exp = np.zeros_like(a.rgb)
    for ch in range(3):
        pv = pal[a.material, ch]
        exp[..., ch] = np.vectorize(orc.quantise)(pv, I[perm[np.minimum(a.face, 6)]])
    np.testing.assert_array_equal(c.rgb[hit], exp[hit])


def test_mirror_in_x_flips_the_image(orc):
    X, Y, Z = 12, 9, 6
    rng, vox, pal = _arena(12, (X, Y, Z))
    cams = np.array([[3.5, 4.5, 1.5, 0.25, 0.125], [7.25, 2.75, 2.5, 2.0, -0.375]], np.float32)
    mir = vox[:, :, ::-1].copy()
    cams_m = cams.copy()
    cams_m[:, 0] = X - cams[:, 0]
    cams_m[:, 3] = np.float32(np.pi) - cams[:, 3]
    a = _render_world(orc, (X, Y, Z), vox, pal, cams, light_dir=(0.0, 0.0, 1.0))
    b = _render_world(orc, (X, Y, Z), mir, pal, cams_m, light_dir=(0.0, 0.0, 1.0))
    ok = (a.edge_margin > 1e-5) & (b.edge_margin[:, :, ::-1] > 1e-5)
    assert ok.mean() > 0.97
    np.testing.assert_array_equal(a.material[ok], b.material[:, :, ::-1][ok])
    np.testing.assert_allclose(a.depth[ok], b.depth[:, :, ::-1][ok], rtol=2e-5)
    np.testing.assert_array_equal(a.rgb[ok], b.rgb[:, :, ::-1][ok])


def test_integer_translation_inside_a_larger_grid(orc):
    X, Y, Z = 8, 7, 5
    rng, vox, pal = _arena(13, (X, Y, Z))
    big = np.zeros((Z + 3, Y + 5, X + 4), np.uint8)
    big[2:2 + Z, 1:1 + Y, 3:3 + X] = vox
    cams = np.array([[3.5, 4.5, 1.5, 0.5, 0.25], [6.25, 2.75, 2.5, 4.0, -0.5]], np.float32)
    cams_b = cams.copy()
    cams_b[:, :3] += np.array([3, 1, 2], np.float32)
    a = _render_world(orc, (X, Y, Z), vox, pal, cams)
    b = _render_world(orc, (X + 4, Y + 5, Z + 3), big, pal, cams_b)
    np.testing.assert_array_equal(a.material, b.material)
    np.testing.assert_array_equal(a.face, b.face)
    np.testing.assert_array_equal(a.rgb, b.rgb)
    np.testing.assert_allclose(a.depth, b.depth, rtol=1e-12)
    hit = a.hit_index >= 0
    k, rem = np.divmod(a.hit_index[hit], X * Y)
    j, i = np.divmod(rem, X)
    np.testing.assert_array_equal(b.hit_index[hit], ((k + 2) * (Y + 5) + j + 1) * (X + 4) + i + 3)


# --------------------------------------------------------------------------- quantisation
def test_quantisation_exhaustive_vs_exact_rationals(orc):
    """All 256 palette values x the seven default intensities (and a few others) against
    round-half-up of the exact rational product."""
    I_default = orc.OracleBatch(1, 1, (2, 2, 2), 8, 8, 1).face_intensity()
    extra = np.array([0.0, 1.0, 0.5, 0.999, 1.2], np.float32)
    near_ties = off_by_one = 0
    for I in list(I_default) + list(extra):
        fi = Fraction(float(I))
        for v in range(256):
            exact = Fraction(v) * fi + Fraction(1, 2)
            want = min(255, int(exact))                       # floor of a non-negative rational
            got = orc.quantise(v, float(I))
            dist = abs(exact - round(exact))
            if dist > Fraction(1, 1 << 14):
                assert got == want, (v, float(I), got, want)
            else:
                # the exact product lies within float32 rounding of a .5 boundary (e.g. 0.3f * 5k):
                # either neighbour is a correct float32 result
                near_ties += 1
                off_by_one += got != want
                assert abs(got - want) <= 1
    assert near_ties < 300 and off_by_one <= near_ties // 4


# --------------------------------------------------------------------------- conventions / side channels
def test_observation_order_and_own_body(orc):
    """Observation o = env*A + agent; each camera ignores its own 1x1x2 body and sees the others'."""
    X, Y, Z = 10, 10, 6
    vox = np.zeros((2, Z, Y, X), np.uint8)
    vox[:, 0] = 1
    pal = np.zeros((2, 4, 3), np.uint8)
    pal[0, 1:] = [(10, 10, 10), (250, 0, 0), (0, 250, 0)]
    pal[1, 1:] = [(20, 20, 20), (0, 0, 250), (250, 250, 0)]
    # env e: agent 0 at (2,5), agent 1 at (7,5), looking at each other; bodies use materials 2 and 3
    for e in range(2):
        vox[e, 1:3, 5, 2] = 2
        vox[e, 1:3, 5, 7] = 3
    cams = np.array([[2.5, 5.5, 1.5, 0.0, 0.0], [7.5, 5.5, 1.5, np.pi, 0.0]] * 2, np.float32)
    selfv = np.array([(1 * Y + 5) * X + 2, (1 * Y + 5) * X + 7] * 2, np.int32)
    b = orc.OracleBatch(2, 2, (X, Y, Z), W, H, 3)
    b.upload_worlds(vox, pal)
    b.set_cameras(cams, selfv)
    out = b.render()
    centre = (H // 2, W // 2)
    assert out.material[0][centre] == 3 and out.material[1][centre] == 2
    assert out.material[2][centre] == 3 and out.material[3][centre] == 2
    np.testing.assert_allclose(out.depth[:, centre[0], centre[1]], 4.5, rtol=1e-6)
    # env 1 uses env 1's palette: face +x... agent 0 looks along +x and enters the -x face (unlit)
    assert tuple(out.rgb[2][centre]) == (75, 75, 0) and tuple(out.rgb[0][centre]) == (0, 75, 0)
    # looking steeply up, the ray leaves through the UPPER voxel of the own body: it must be invisible too
    up = cams.copy()
    up[:, 4] = 1.2
    b.set_cameras(up, selfv)
    out_up = b.render()
    assert (out_up.hit_index[:, H // 2, W // 2] == -1).all() and (out_up.face[:, H // 2, W // 2] == 255).all()
    # without the own-body rule every camera would be inside a solid: face 6 everywhere
    b.set_cameras(cams, None)
    out2 = b.render()
    assert (out2.face == 6).all() and (out2.depth == 0).all() and (out2.hit_index[0] == selfv[0]).all()


def test_step_count_and_termination_bound(orc):
    wl = synth.generate(0)
    s = wl.spec
    b = orc.OracleBatch(s.num_envs, s.agents_per_env, s.grid, s.width, s.height, s.num_materials)
    b.upload_worlds(wl.voxels, wl.palette)
    b.set_cameras(wl.cameras[0])
    out = b.render()
    assert out.steps.max() <= sum(s.grid)
    assert (out.steps[out.hit_index >= 0] >= 1).all()      # camera cells are empty, so >= 1 crossing


def test_vertical_and_axis_parallel_rays_terminate(orc):
    """Directions with exact zeros (never step on that axis) and straight up/down."""
    grid = (6, 6, 6)
    vox = np.zeros((6, 6, 6), np.uint8)
    vox[0] = 1
    vox[5, 2, 2] = 2
    pal = np.full((3, 3), 200, np.uint8)
    # 2x2 image with a tiny fov keeps rays nearly parallel to the view axis
    b = orc.OracleBatch(1, 3, grid, 2, 2, 2, hfov_rad=1e-3)
    b.upload_worlds(vox[None], pal[None])
    b.set_cameras(np.array([[2.5, 2.5, 2.5, 0.0, -np.pi / 2], [2.5, 2.5, 2.5, 0.0, np.pi / 2],
                            [2.5, 2.5, 2.5, 0.0, 0.0]], np.float32))
    out = b.render()
    assert (out.face[0] == 5).all() and np.allclose(out.depth[0], 1.5)
    assert (out.face[1] == 4).all() and np.allclose(out.depth[1], 2.5) and (out.material[1] == 2).all()
    assert (out.hit_index[2] == -1).all()


def test_exact_zero_direction_components(orc):
    """A 1x1 image has sx = sy = 0, so with yaw = pitch = 0 the ray is exactly (1,0,0): two axes
    never step.  It must still find the wall ahead, and miss when there is none."""
    grid = (6, 6, 6)
    vox = np.zeros((6, 6, 6), np.uint8)
    vox[2, 2, 5] = 1
    pal = np.full((2, 3), 100, np.uint8)
    b = orc.OracleBatch(1, 2, grid, 1, 1, 1)
    b.upload_worlds(vox[None], pal[None])
    b.set_cameras(np.array([[0.5, 2.5, 2.5, 0.0, 0.0], [0.5, 3.5, 2.5, 0.0, 0.0]], np.float32))
    np.testing.assert_array_equal(b.pixel_rays(0)[0, 0], [1.0, 0.0, 0.0])
    out = b.render()
    assert out.hit_index[0, 0, 0] == (2 * 6 + 2) * 6 + 5 and out.depth[0, 0, 0] == 4.5 and out.face[0, 0, 0] == 0
    assert out.hit_index[1, 0, 0] == -1 and out.steps[1, 0, 0] == 6


def test_sparse_edits_equal_a_fresh_upload(orc):
    """mvo_update_voxels is pinned by the plain definition of what an edit is: rendering after the
    edits equals rendering a batch that received the edited grids wholesale."""
    rng = np.random.default_rng(77)
    grid = (9, 7, 5)
    vox, pal = synth.random_world(rng, 3, grid, 0.2, 6)
    vox[:, 0] = 2
    cams = synth.random_cameras(rng, 6, grid, margin=0.0, max_pitch=0.7)
    after = vox.copy()
    flip = rng.random(size=vox.shape) < 0.03
    after[flip] = np.where(vox[flip] == 0, rng.integers(1, 7, size=int(flip.sum()), dtype=np.uint8), 0)
    env, idx, mat = synth.grid_edits(vox, after)
    assert env.size == int(flip.sum()) and (mat == after.reshape(3, -1)[env, idx]).all()
    a = orc.OracleBatch(3, 2, grid, 48, 32, 6)
    a.upload_worlds(vox, pal)
    a.update_voxels(env, idx, mat)
    a.set_cameras(cams)
    b = orc.OracleBatch(3, 2, grid, 48, 32, 6)
    b.upload_worlds(after, pal)
    b.set_cameras(cams)
    ra, rb = a.render(), b.render()
    for name in ("rgb", "depth", "material", "hit_index", "face"):
        np.testing.assert_array_equal(getattr(ra, name), getattr(rb, name))
    assert not np.array_equal(ra.hit_index, _render_with(orc, grid, vox, pal, cams).hit_index)   # the edits are visible
    with pytest.raises(ValueError):
        a.update_voxels(np.array([3], np.int32), np.array([0], np.int32), np.array([1], np.uint8))
    with pytest.raises(ValueError):
        a.update_voxels(np.array([0], np.int32), np.array([9 * 7 * 5], np.int32), np.array([1], np.uint8))
    with pytest.raises(ValueError):
        a.update_voxels(np.array([0], np.int32), np.array([0], np.int32), np.array([7], np.uint8))


def _render_with(orc, grid, vox, pal, cams):
    b = orc.OracleBatch(vox.shape[0], cams.shape[0] // vox.shape[0], grid, 48, 32, pal.shape[1] - 1)
    b.upload_worlds(vox, pal)
    b.set_cameras(cams)
    return b.render()


def test_indicator_bar_closed_form(orc):
    """The bar's filled width is round-half-up(fraction * width) columns, clamped; nothing outside the
    rectangle changes; inactive environments are skipped."""
    b = orc.OracleBatch(3, 2, (4, 4, 4), 64, 40, 2)
    fractions = np.array([0.0, 1.0, 0.5, 0.28, 0.999, 1.7], np.float32)
    rgb = np.full((6, 40, 64, 3), 9, np.uint8)
    x, y, w, h = 5, 3, 20, 4
    b.draw_bars(rgb, fractions, x, y, w, h, (250, 10, 20), (1, 2, 3), active=np.array([1, 1, 0], np.uint8))
    for o, f in enumerate(fractions):
        bar = rgb[o, y:y + h, x:x + w]
        outside = rgb[o].copy()
        outside[y:y + h, x:x + w] = 9
        assert (outside == 9).all()
        if o >= 4:                                    # environment 2 is inactive
            assert (bar == 9).all()
            continue
        want = min(w, max(0, int(Fraction(float(f)) * w + Fraction(1, 2))))
        assert (bar[:, :want] == np.array((250, 10, 20), np.uint8)).all()
        assert (bar[:, want:] == np.array((1, 2, 3), np.uint8)).all()
        assert {0: 0, 1: 20, 2: 10, 3: 6}[o] == want          # 0.28 * 20 = 5.6 rounds up to 6
    with pytest.raises(ValueError):
        b.draw_bars(rgb, fractions, 60, 3, 20, 4, (0, 0, 0), (0, 0, 0))      # sticks out of the image


def test_overlay_rectangles_paint_in_list_order(orc):
    """Solid primitives against NumPy slice assignment in the same order: later rectangles cover earlier ones,
    nothing outside any rectangle changes, inactive environments are skipped, bad lists are refused."""
    b = orc.OracleBatch(2, 2, (4, 4, 4), 64, 40, 2)
    rects = [(2, 3, 30, 20, (200, 1, 2), 0, (0, 0, 0), 0),
             (10, 10, 40, 12, (3, 210, 4), 0, (0, 0, 0), 0),       # overlaps the first
             (25, 0, 6, 40, (5, 6, 220), 0, (0, 0, 0), 0),         # a full-height stripe over both
             (63, 39, 1, 1, (7, 8, 9), 0, (0, 0, 0), 0)]           # the last pixel of the image
    rgb = np.full((4, 40, 64, 3), 77, np.uint8)
    b.draw_overlay(rgb, rects, active=np.array([1, 0], np.uint8))
    want = np.full((40, 64, 3), 77, np.uint8)
    for x, y, w, h, colour, *_ in rects:
        want[y:y + h, x:x + w] = colour
    assert (want[11, 26] == (5, 6, 220)).all() and (want[11, 12] == (3, 210, 4)).all() and (want[4, 4] == (200, 1, 2)).all()
    np.testing.assert_array_equal(rgb[0], want)
    np.testing.assert_array_equal(rgb[1], want)
    assert (rgb[2:] == 77).all()                      # environment 1 is inactive
    for bad in ([(60, 3, 20, 4, (0, 0, 0), 0, (0, 0, 0), 0)],       # sticks out of the image
                [(0, 0, 4, 4, (0, 0, 0), 3, (0, 0, 0), 0)],        # no such kind
                [(0, 0, 4, 4, (0, 0, 0), 1, (0, 0, 0), 0)]):       # a gauge without values
        with pytest.raises(ValueError):
            b.draw_overlay(rgb, bad)
    with pytest.raises(ValueError):                                # a gauge whose value column does not exist
        b.draw_overlay(rgb, [(0, 0, 4, 4, (0, 0, 0), 1, (0, 0, 0), 2)], values=np.zeros((4, 2), np.float32))


def test_overlay_gauges_closed_form(orc):
    """A gauge shows round-half-up(value * extent) columns from the left (kind 1) or rows from the bottom (kind 2),
    clamped to the rectangle, with exact rationals as the reference; a rightward gauge is the indicator bar."""
    b = orc.OracleBatch(3, 2, (4, 4, 4), 64, 40, 2)
    values = np.array([[0.0, 1.0], [1.0, 0.0], [0.5, 0.28], [0.28, 0.5], [0.999, -3.0], [1.7, 0.126]], np.float32)
    front, rest = (250, 10, 20), (1, 2, 3)
    x, y, w, h = 5, 3, 20, 25
    rects = [(x, y, w, h, front, 2, rest, 1),                      # upward gauge on column 1 of the values
             (40, 30, 20, 4, front, 1, rest, 0)]                   # rightward gauge on column 0
    rgb = np.full((6, 40, 64, 3), 9, np.uint8)
    b.draw_overlay(rgb, rects, values=values)
    bars = np.full((6, 40, 64, 3), 9, np.uint8)
    b.draw_bars(bars, values[:, 0].copy(), 40, 30, 20, 4, front, rest)
    seen = set()
    for o in range(6):
        rows = min(h, max(0, int(Fraction(float(values[o, 1])) * h + Fraction(1, 2))))
        seen.add(rows)
        up = rgb[o, y:y + h, x:x + w]
        assert (up[h - rows:] == np.array(front, np.uint8)).all()          # the lowest rows
        assert (up[:h - rows] == np.array(rest, np.uint8)).all()
        np.testing.assert_array_equal(rgb[o, 30:34, 40:60], bars[o, 30:34, 40:60])
        outside = rgb[o].copy()
        outside[y:y + h, x:x + w] = 9
        outside[30:34, 40:60] = 9
        assert (outside == 9).all()
    assert seen == {25, 0, 7, 13, 3}                  # 0.28 * 25 = 7 exactly, 0.5 * 25 = 12.5 rounds up, 0.126 * 25 = 3.15


def test_pitched_camera_floor_landing_points(orc):
    """Closed form for a pitched, yawed camera over a solid floor: the pixel ray
    d = F + sx*R + sy*U with F = (cp*cy, cp*sy, sp), R = tx*(sy_, -cy_, 0), U = ty*(-sp*cy, -sp*sy, cp)
    reaches the floor plane z = 1 at t = (1 - Pz)/d_z and lands in the cell under P + t*d.  Pins the
    horizontal components of the up vector and the pitch sign, which the unpitched pins cannot see."""
    grid = (40, 40, 6)
    vox = np.zeros((6, 40, 40), np.uint8)
    vox[0] = 1
    pal = np.array([[0, 0, 0], [200, 200, 200]], np.uint8)
    yaw, pitch = 0.9, -0.45
    cam = np.array([[20.5, 20.5, 2.5, yaw, pitch]], np.float32)
    _, out = _single(orc, grid, vox, pal, cam)
    yaw, pitch = float(cam[0, 3]), float(cam[0, 4])
    cy_, sy_, cp, sp = np.cos(yaw), np.sin(yaw), np.cos(pitch), np.sin(pitch)
    tx = np.tan(0.5 * HFOV)
    ty = tx * H / W
    F = np.array([cp * cy_, cp * sy_, sp])
    R = tx * np.array([sy_, -cy_, 0.0])
    U = ty * np.array([-sp * cy_, -sp * sy_, cp])
    c = np.arange(W)
    r = np.arange(H)
    sx = ((2 * c + 1 - W) / W)[None, :, None]
    sy = ((H - 2 * r - 1) / H)[:, None, None]
    d = F + sx * R + sy * U                                    # [H,W,3]
    P = np.array([20.5, 20.5, 2.5])
    down = d[..., 2] < -1e-9
    t = np.where(down, (1.0 - P[2]) / np.where(down, d[..., 2], -1.0), 1e9)
    land = P + t[..., None] * d
    inside = down & (land[..., 0] > 0) & (land[..., 0] < 40) & (land[..., 1] > 0) & (land[..., 1] < 40)
    margin = np.abs(land[..., :2] - np.round(land[..., :2])).min(axis=-1)
    sure = inside & (margin > 1e-4)
    assert sure.sum() > 4000
    ij = np.floor(land[..., :2]).astype(int)
    np.testing.assert_array_equal(out.hit_index[0][sure], (ij[..., 1] * 40 + ij[..., 0])[sure])
    np.testing.assert_allclose(out.depth[0][sure], t[sure], rtol=2e-6)
    assert (out.face[0][sure] == 5).all()
    clear_miss = ~down | (~inside & (np.abs(land[..., :2] - 20).max(axis=-1) > 20.01))
    assert (out.hit_index[0][clear_miss] == -1).all()


def test_edge_margin_flags_ties_at_the_grid_boundary(orc):
    """The margin side channel must mark a ray as a tie wherever its fate hangs on rounding: also when the
    choice is between leaving the grid and entering the last voxel before the boundary.  A 1x1 image looks
    along yaw exactly (sx = sy = 0); the ray from (6.5, 3.5) towards the corner (8, 6) either leaves through
    x = 8 or enters voxel (7, 6) through y = 6.  Slightly turned either way it does one or the other, and
    both times it passes the corner within 5e-5: the margin must say so.  A ray aimed well away from the
    corner must keep a large margin."""
    grid = (8, 8, 4)
    vox = np.zeros((4, 8, 8), np.uint8)
    vox[1, 6, 7] = 1
    pal = np.full((2, 3), 100, np.uint8)
    yaw = np.arctan2(2.5, 1.5)
    cams = np.array([[6.5, 3.5, 1.5, yaw - 2e-6, 0.0], [6.5, 3.5, 1.5, yaw + 2e-6, 0.0],
                     [6.5, 3.5, 1.5, yaw - 0.2, 0.0], [6.5, 3.5, 1.5, yaw + 0.1, 0.0]], np.float32)
    b = orc.OracleBatch(1, 4, grid, 1, 1, 1)
    b.upload_worlds(vox[None], pal[None])
    b.set_cameras(cams)
    out = b.render()
    hit = out.hit_index[:, 0, 0]
    assert hit[0] == -1 and hit[1] == (1 * 8 + 6) * 8 + 7, hit          # one leaves, one enters
    assert out.edge_margin[0, 0, 0] < 5e-5 and out.edge_margin[1, 0, 0] < 5e-5
    assert hit[2] == -1 and out.edge_margin[2, 0, 0] > 0.01             # clear miss
    assert hit[3] == (1 * 8 + 6) * 8 + 7 and out.edge_margin[3, 0, 0] > 0.01   # clear hit


def test_edge_margin_flags_a_ray_that_passes_the_grid_by_at_its_rim(orc):
    """A camera outside the grid: the ray towards the vertical rim x = 0, y = 0 of the grid either enters the
    corner voxel through the face x = 0 or passes the whole grid by.  Turned a hair either way it does one or the
    other, and both are ties: the one that enters has a small margin from its first crossing, the one that passes
    by must have one too (how far outside the face's rectangle it meets the plane x = 0).  A ray that passes
    the rim at a distance keeps that distance as its margin, one that enters through the middle of the face a large one."""
    grid = (4, 6, 3)
    vox = np.zeros((3, 6, 4), np.uint8)
    vox[1, 0, 0] = 1
    pal = np.full((2, 3), 100, np.uint8)
    P = (-2.0, 3.0, 1.5)
    yaw = np.arctan2(-3.0, 2.0)                      # from (-2, 3) to the rim at (0, 0)
    turned = yaw - 0.1                               # meets x = 0 at y = 3 + 2 tan(turned) < 0
    cams = np.array([[*P, yaw + 2e-6, 0.0], [*P, yaw - 2e-6, 0.0], [*P, turned, 0.0], [*P, yaw + 0.5, 0.0]], np.float32)
    b = orc.OracleBatch(1, 4, grid, 1, 1, 1)
    b.upload_worlds(vox[None], pal[None])
    b.set_cameras(cams)
    out = b.render()
    hit, m = out.hit_index[:, 0, 0], out.edge_margin[:, 0, 0]
    assert hit[0] == (1 * 6 + 0) * 4 + 0 and hit[1] == -1, hit               # one enters, one passes by
    assert m[0] < 5e-5 and m[1] < 5e-5, m
    y_at_plane = 3.0 + 2.0 * np.tan(np.float64(np.float32(turned)))
    assert hit[2] == -1 and abs(m[2] - (-y_at_plane)) < 1e-5, (m[2], y_at_plane)
    assert hit[3] == -1 and m[3] > 0.02          # through the middle of the face and out again past the corner voxel


def _margin_by_plane_enumeration(P, d, t_begin, t_end, dims):
    """The margin side channel written out from its definition, with no traversal: every integer plane of every
    axis that the ray reaches at a parameter t_begin <= t <= t_end (t > 0) is a crossing; at each crossing, the
    distance from the crossing point to the nearest integer along each of the two OTHER axes; the minimum over
    all of them."""
    best = np.inf
    for a in range(3):
        if d[a] == 0.0:
            continue
        for plane in range(0, dims[a] + 1):
            t = (plane - P[a]) / d[a]
            if not (t > 0.0 and t_begin * (1 - 1e-12) <= t <= t_end * (1 + 1e-12)):
                continue
            for o in range(3):
                if o == a:
                    continue
                q = P[o] + t * d[o]
                best = min(best, abs(q - np.rint(q)))
    return best


def test_edge_margin_equals_plane_enumeration(orc):
    """edge_margin against its definition, enumerated plane by plane in Python: random small worlds, cameras
    inside and outside the grid, every pixel.  The crossings run from the one that takes the ray into the grid
    (cameras outside) up to the hit, or for a miss up to and including the crossing through the grid boundary.
    A margin that skips crossings, uses the wrong axes or the wrong parameter differs on almost every pixel."""
    rng = np.random.default_rng(77)
    w, h = 16, 9
    checked = outside_checked = passed_by = 0
    for trial in range(8):
        grid = (int(rng.integers(3, 9)), int(rng.integers(3, 9)), int(rng.integers(2, 5)))
        vox, pal = synth.random_world(rng, 1, grid, float(rng.uniform(0.02, 0.2)), 3)
        cams = synth.random_cameras(rng, 2, grid, margin=0.0)
        cams[:, :3] = np.clip(cams[:, :3], 0.05, np.array(grid, np.float32) - 0.05)
        if trial >= 4:                        # outside the grid, looking roughly at its centre
            away = rng.uniform(0.3, 2.0)
            cams[:, 0] = -away
            cams[:, 3] = rng.uniform(-0.5, 0.5, 2)
        b, out = _single(orc, grid, vox[0], pal[0], cams, w=w, h=h)
        for a in range(2):
            P = b.camera_record(a)[:3].astype(np.float64)
            rays = b.pixel_rays(a).astype(np.float64)
            for r in range(h):
                for c in range(w):
                    d = rays[r, c]
                    lo = [min((0.0 - P[k]) / d[k], (grid[k] - P[k]) / d[k]) for k in range(3) if d[k] != 0.0]
                    hi = [max((0.0 - P[k]) / d[k], (grid[k] - P[k]) / d[k]) for k in range(3) if d[k] != 0.0]
                    t_begin, t_exit = max(max(lo), 0.0), min(hi)
                    got = out.edge_margin[a, r, c]
                    if t_begin > t_exit:
                        # never enters the grid: the margin is how far outside the rectangle of the boundary face
                        # the ray meets that face's plane (the plane of the last slab it enters)
                        assert out.hit_index[a, r, c] == -1
                        if t_exit < 0.0:                                     # the grid lies behind the camera
                            assert got == np.inf
                            continue
                        k_in = int(np.argmax([min((0.0 - P[k]) / d[k], (grid[k] - P[k]) / d[k]) if d[k] != 0.0
                                              else -np.inf for k in range(3)]))
                        q = P + t_begin * d
                        want = max(max(-q[o], q[o] - grid[o], 0.0) for o in range(3) if o != k_in)
                        assert abs(got - want) <= 1e-9, (trial, a, r, c, got, want)
                        passed_by += 1
                        continue
                    if out.hit_index[a, r, c] >= 0:
                        if out.steps[a, r, c] == 0 and t_begin == 0.0:
                            assert got == np.inf                             # camera inside a solid: no crossing
                            continue
                        t_end = out.t[a, r, c]
                    else:
                        t_end = t_exit
                    want = _margin_by_plane_enumeration(P, d, t_begin, t_end, grid)
                    if want < 1e-9:                                          # exact ties: order of crossings is open
                        continue
                    assert abs(got - want) <= 1e-9, (trial, a, r, c, got, want)
                    checked += 1
                    outside_checked += int(t_begin > 0.0)
    assert checked > 1500 and outside_checked > 300 and passed_by > 100, (checked, outside_checked, passed_by)


def test_edge_margin_flags_a_grazed_edge_inside_the_grid(orc):
    """A ray that only grazes a voxel edge in the MIDDLE of its path and then goes on to a clear hit is a tie as
    well: turned a hair one way it enters the pillar, turned the other way it passes the pillar's corner and hits
    the far wall.  Both must carry a margin below 5e-5 (for the second the near-tie is an early crossing, not the
    last one); rays aimed well to either side keep a large margin."""
    grid = (8, 8, 4)
    vox = np.zeros((4, 8, 8), np.uint8)
    vox[1, 3, 4] = 1                      # pillar voxel (i=4, j=3): its corner (x=4, y=4) is the grazed edge
    vox[1, :, 7] = 2                      # far wall x = 7
    pal = np.full((3, 3), 100, np.uint8)
    px, py = 1.3, 1.7
    yaw = np.arctan2(4.0 - py, 4.0 - px)
    cams = np.array([[px, py, 1.5, yaw - 4e-6, 0.0], [px, py, 1.5, yaw + 4e-6, 0.0],
                     [px, py, 1.5, yaw - 0.15, 0.0], [px, py, 1.5, yaw + 0.11, 0.0]], np.float32)
    b = orc.OracleBatch(1, 4, grid, 1, 1, 2)
    b.upload_worlds(vox[None], pal[None])
    b.set_cameras(cams)
    out = b.render()
    hit, mat = out.hit_index[:, 0, 0], out.material[:, 0, 0]
    pillar = (1 * 8 + 3) * 8 + 4
    assert hit[0] == pillar and mat[1] == 2, (hit, mat)                  # one enters the pillar, one reaches the wall
    assert out.edge_margin[0, 0, 0] < 5e-5 and out.edge_margin[1, 0, 0] < 5e-5, out.edge_margin[:, 0, 0]
    assert out.steps[1, 0, 0] > out.steps[0, 0, 0] + 2                   # the graze is not the wall ray's last crossing
    assert hit[2] == pillar and out.edge_margin[2, 0, 0] > 0.01          # clear hit on the pillar
    assert mat[3] == 2 and out.edge_margin[3, 0, 0] > 0.01               # clear pass


def test_single_pixel_entry_point_equals_the_full_render(orc):
    """mvo_render_pixels (chosen pixels one by one, used for sampled comparisons at full batch size) returns,
    field by field, what mvo_render holds at the same (observation, row, column)."""
    wl = synth.generate(0)
    s = wl.spec
    b = orc.OracleBatch(s.num_envs, s.agents_per_env, s.grid, s.width, s.height, s.num_materials)
    b.upload_worlds(wl.voxels, wl.palette)
    b.set_cameras(wl.cameras[0])
    full = b.render()
    rng = np.random.default_rng(5)
    n = 4000
    obs = rng.integers(0, s.num_obs, n).astype(np.int32)
    row = rng.integers(0, s.height, n).astype(np.int32)
    col = rng.integers(0, s.width, n).astype(np.int32)
    row[:4], col[:4] = [0, 0, s.height - 1, s.height - 1], [0, s.width - 1, 0, s.width - 1]
    px = b.render_pixels(obs, row, col)
    for name in ("rgb", "depth", "material", "hit_index", "face", "steps", "edge_margin", "t"):
        np.testing.assert_array_equal(getattr(px, name), getattr(full, name)[obs, row, col], err_msg=name)
    with pytest.raises(ValueError):
        b.render_pixels(np.array([s.num_obs], np.int32), np.array([0], np.int32), np.array([0], np.int32))
