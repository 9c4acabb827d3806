"""GPU parity: the HIP library through its C ABI against the CPU oracle, element by element, on the
same seeded inputs.  Needs a real MI355X; run with ``-m gpu``."""
import ctypes as C

import numpy as np
import pytest

from paper_2107_08170_amd import binding, synth
from tests import parity

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def lib():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU (torch.cuda.is_available() is False)")
    return binding.load_library()          # raises if libmv.so is missing: there is no fallback


def _stream():
    return torch.cuda.current_stream().cuda_stream


class GpuRender:
    """Owns the output tensors of one batch and renders into them."""

    def __init__(self, batch: binding.Batch, W, H, aux=True):
        n = batch.num_obs
        dev = torch.device("cuda", 0)
        self.batch = batch
        self.rgb = torch.empty((n, H, W, 3), dtype=torch.uint8, device=dev)
        self.depth = torch.empty((n, H, W), dtype=torch.float32, device=dev)
        self.aux = aux
        if aux:
            self.material = torch.empty((n, H, W), dtype=torch.uint8, device=dev)
            self.hit = torch.empty((n, H, W), dtype=torch.int32, device=dev)
            self.face = torch.empty((n, H, W), dtype=torch.uint8, device=dev)

    def render(self):
        # poison the outputs so that an unwritten pixel cannot pass by accident
        self.rgb.fill_(7)
        self.depth.fill_(-1.0)
        if self.aux:
            self.material.fill_(254); self.hit.fill_(-7); self.face.fill_(9)
            self.batch.render(self.rgb, self.depth, self.material, self.hit, self.face, stream=_stream())
        else:
            self.batch.render(self.rgb, self.depth, stream=_stream())
        torch.cuda.synchronize()

    def numpy(self, obs=None) -> parity.GpuOut:
        sel = slice(None) if obs is None else torch.as_tensor(obs, device=self.rgb.device)
        g = parity.GpuOut(self.rgb[sel].cpu().numpy(), self.depth[sel].cpu().numpy())
        if self.aux:
            g.material = self.material[sel].cpu().numpy()
            g.hit_index = self.hit[sel].cpu().numpy()
            g.face = self.face[sel].cpu().numpy()
        return g


def _oracle_for(orc, spec, voxels, palette, cams, self_voxel=None, **kw):
    b = orc.OracleBatch(spec.num_envs, spec.agents_per_env, spec.grid, spec.width, spec.height,
                        spec.num_materials, **kw)
    b.upload_worlds(voxels, palette)
    b.set_cameras(cams, self_voxel)
    return b


def _gpu_for(spec, voxels, palette, cams, self_voxel=None, device_src=True, aux=True, tiles_per_block=0, **kw):
    batch = binding.Batch(spec.num_envs, spec.agents_per_env, spec.grid, spec.num_materials, spec.width,
                          spec.height, tiles_per_block=tiles_per_block, **kw)
    if device_src:
        batch.upload_worlds(torch.from_numpy(voxels).cuda(), torch.from_numpy(palette).cuda(), stream=_stream())
        batch.set_cameras(torch.from_numpy(np.ascontiguousarray(cams)).cuda(),
                          None if self_voxel is None else torch.from_numpy(np.ascontiguousarray(self_voxel)).cuda(),
                          stream=_stream())
        torch.cuda.synchronize()        # the temporaries above are released right after this line
    else:
        batch.upload_worlds(voxels, palette, stream=_stream())
        batch.set_cameras(np.ascontiguousarray(cams), self_voxel, stream=_stream())
    return GpuRender(batch, spec.width, spec.height, aux=aux)


def _obs_sample(spec, count):
    step = max(1, spec.num_obs // count)
    return np.arange(0, spec.num_obs, step, dtype=np.int64)[:count]


def _compare_sampled(orc, ob, run, obs_ids, label, threads=16):
    stats = []
    # contiguous runs keep the oracle call count low
    for o in obs_ids:
        ref = ob.render(first_obs=int(o), count=1, threads=1)
        stats.append(parity.compare(run.numpy([int(o)]), ref, label=f"{label} obs {int(o)}"))
    return stats


def _compare_all(ob, run, label, chunk=512, threads=16):
    """Every observation of the batch against the oracle, in chunks that keep the oracle's output small.
    Returns the totals over the batch."""
    n = run.rgb.shape[0]
    pixels = differ = 0
    worst_depth = 0.0
    for o0 in range(0, n, chunk):
        c = min(chunk, n - o0)
        ref = ob.render(first_obs=o0, count=c, threads=threads)
        st = parity.compare(run.numpy(np.arange(o0, o0 + c)), ref, label=f"{label} obs {o0}..{o0 + c - 1}")
        pixels += st["pixels"]; differ += st["differ"]
        worst_depth = max(worst_depth, st["max_depth_rel"])
    return {"pixels": pixels, "differ": differ, "max_depth_rel": worst_depth}


# ------------------------------------------------------------------------------------------ configs 0, 1
@pytest.mark.parametrize("device_src", [True, False])
def test_config0_full_parity(lib, orc, device_src):
    wl = synth.generate(0)
    ob = _oracle_for(orc, wl.spec, wl.voxels, wl.palette, wl.cameras[0])
    run = _gpu_for(wl.spec, wl.voxels, wl.palette, wl.cameras[0], device_src=device_src)
    run.render()
    st = parity.compare(run.numpy(), ob.render(), label="cfg0")
    assert st["pixels"] == 4 * 72 * 128
    assert st["colour_exact_fraction"] == 1.0       # the colour table uses the oracle's two roundings


def test_config1_full_parity_and_launch_shapes(lib, orc):
    wl = synth.generate(1)
    ob = _oracle_for(orc, wl.spec, wl.voxels, wl.palette, wl.cameras[0])
    ref = ob.render(threads=16)
    first = None
    for tpb in (0, 1, 5, 16, 144, 100000):
        run = _gpu_for(wl.spec, wl.voxels, wl.palette, wl.cameras[0], tiles_per_block=tpb)
        run.render()
        g = run.numpy()
        parity.compare(g, ref, label=f"cfg1 tiles_per_block={tpb}")
        if first is None:
            first = g
        else:                               # the launch shape must not change a single bit
            for name in ("rgb", "depth", "material", "hit_index", "face"):
                np.testing.assert_array_equal(getattr(g, name).view(np.uint8), getattr(first, name).view(np.uint8))
    # colour+depth-only launch (the one the benchmark times) writes the same bits
    run = _gpu_for(wl.spec, wl.voxels, wl.palette, wl.cameras[0], aux=False)
    run.render()
    g = run.numpy()
    np.testing.assert_array_equal(g.rgb, first.rgb)
    np.testing.assert_array_equal(g.depth.view(np.uint32), first.depth.view(np.uint32))


def test_config1_certificate_against_the_scene(lib, orc):
    """Independent of the oracle's traversal: hit points lie on the claimed faces and brute force
    finds nothing nearer."""
    wl = synth.generate(1)
    ob = _oracle_for(orc, wl.spec, wl.voxels, wl.palette, wl.cameras[0])
    run = _gpu_for(wl.spec, wl.voxels, wl.palette, wl.cameras[0])
    run.render()
    rng = np.random.default_rng(3)
    obs_ids = [0, 5, 333, 1023]
    g = run.numpy(obs_ids)
    checked = 0
    for local, o in enumerate(obs_ids):
        checked += parity.certificate(orc, ob, wl.voxels[o // wl.spec.agents_per_env], o, g, local, rng, samples=150)
    assert checked > 300


# ------------------------------------------------------------------------------------------ config 2
def test_config2_full_size_first_and_last_step(lib, orc):
    """4096 envs x 2 agents at full size, in the launch configuration the benchmark times
    (device-resident inputs, automatic launch shape, colour+depth only) and once more with the auxiliary
    outputs: every one of the 8192 observations of the first and the last camera set against the oracle."""
    wl = synth.generate(2)
    spec = wl.spec
    vox_d = torch.from_numpy(wl.voxels).cuda()
    pal_d = torch.from_numpy(wl.palette).cuda()
    cams_d = torch.from_numpy(wl.cameras).cuda()            # [100, 8192, 5]
    batch = binding.Batch(spec.num_envs, spec.agents_per_env, spec.grid, spec.num_materials, spec.width, spec.height)
    batch.upload_worlds(vox_d, pal_d, stream=_stream())
    plain = GpuRender(batch, spec.width, spec.height, aux=False)
    full = GpuRender(batch, spec.width, spec.height, aux=True)
    ob = orc.OracleBatch(spec.num_envs, spec.agents_per_env, spec.grid, spec.width, spec.height, spec.num_materials)
    ob.upload_worlds(wl.voxels, wl.palette)
    for step in (0, spec.steps - 1):
        batch.set_cameras(cams_d[step], stream=_stream())
        ob.set_cameras(wl.cameras[step])
        plain.render()
        full.render()
        assert torch.equal(plain.rgb, full.rgb) and torch.equal(plain.depth.view(torch.int32), full.depth.view(torch.int32))
        total = _compare_all(ob, full, f"cfg2 step {step}")
        assert total["pixels"] == spec.num_obs * spec.width * spec.height
        assert total["differ"] <= 5e-4 * total["pixels"]
        # whole-batch properties that hold at any size
        miss = full.hit < 0
        assert bool((full.depth[miss] == 0).all()) and bool((full.depth[~miss] > 0).all())
        assert bool((full.material[~miss] >= 1).all()) and bool((full.material[~miss] <= spec.num_materials).all())
        assert bool((full.face[~miss] <= 5).all()) and bool((full.face[miss] == 255).all())
        assert int(full.hit.max()) < spec.grid[0] * spec.grid[1] * spec.grid[2]


# ------------------------------------------------------------------------------------------ config 3
def test_config3_dynamic_worlds_and_own_bodies(lib, orc):
    wl = synth.generate(3)
    spec = wl.spec
    batch = binding.Batch(spec.num_envs, spec.agents_per_env, spec.grid, spec.num_materials, spec.width, spec.height)
    run = GpuRender(batch, spec.width, spec.height, aux=True)
    ob = orc.OracleBatch(spec.num_envs, spec.agents_per_env, spec.grid, spec.width, spec.height, spec.num_materials)
    pal_d = torch.from_numpy(wl.palette).cuda()
    vox, cams, selfv = wl.voxels, wl.cameras[0], wl.self_voxel[0]
    saw_body = 0
    for step in range(4):
        if step:
            vox, cams, selfv = synth.dynamic_step(wl)
        vox_d = torch.from_numpy(vox).cuda()
        batch.upload_worlds(vox_d, pal_d if step == 0 else None, stream=_stream())     # palette kept after step 0
        batch.set_cameras(torch.from_numpy(cams).cuda(), torch.from_numpy(selfv).cuda(), stream=_stream())
        torch.cuda.synchronize()
        run.render()
        ob.upload_worlds(vox, wl.palette if step == 0 else None)
        ob.set_cameras(cams, selfv)
        _compare_all(ob, run, f"cfg3 step {step}")
        # no camera may see its own body; some cameras do see other agents' bodies or boxes
        hit = run.hit.view(spec.num_obs, -1)
        sv = torch.from_numpy(selfv).cuda().view(-1, 1)
        assert not bool(((hit == sv) | (hit == sv + spec.grid[0] * spec.grid[1])).any())
        saw_body += int((run.face.view(spec.num_obs, -1) == 6).sum())
    assert saw_body == 0        # the own-body rule keeps every camera out of "inside a solid"


def test_config3_sparse_edits_match_full_uploads(lib, orc):
    """Stepping the dynamic workload with mv_update_voxels (only the changed voxels) gives bit for bit
    the frames of re-uploading whole grids, from device-resident and from host edit lists."""
    wl = synth.generate(3, num_envs=128)
    spec = wl.spec
    mk = lambda: binding.Batch(spec.num_envs, spec.agents_per_env, spec.grid, spec.num_materials, spec.width, spec.height)
    full, sparse_d, sparse_h = mk(), mk(), mk()
    runs = [GpuRender(b, spec.width, spec.height, aux=True) for b in (full, sparse_d, sparse_h)]
    ob = orc.OracleBatch(spec.num_envs, spec.agents_per_env, spec.grid, spec.width, spec.height, spec.num_materials)
    vox, cams, selfv = wl.voxels, wl.cameras[0], wl.self_voxel[0]
    for b in (full, sparse_d, sparse_h):
        b.upload_worlds(vox, wl.palette)
    ob.upload_worlds(vox, wl.palette)
    total_edits = 0
    for step in range(5):
        if step:
            prev = vox
            vox, cams, selfv = synth.dynamic_step(wl)
            env, idx, mat = synth.grid_edits(prev, vox)
            total_edits += env.size
            full.upload_worlds(torch.from_numpy(vox).cuda(), None, stream=_stream())
            sparse_d.update_voxels(torch.from_numpy(env).cuda(), torch.from_numpy(idx).cuda(), torch.from_numpy(mat).cuda(),
                                   stream=_stream())
            sparse_h.update_voxels(env, idx, mat, stream=_stream())
            ob.update_voxels(env, idx, mat)
            torch.cuda.synchronize()
        cams_d, self_d = torch.from_numpy(cams).cuda(), torch.from_numpy(selfv).cuda()
        for b in (full, sparse_d, sparse_h):
            b.set_cameras(cams_d, self_d, stream=_stream())
        torch.cuda.synchronize()
        for r in runs:
            r.render()
        for r in runs[1:]:
            for name in ("rgb", "depth", "material", "hit", "face"):
                assert torch.equal(getattr(r, name).view(torch.uint8), getattr(runs[0], name).view(torch.uint8)), (step, name)
        ob.set_cameras(cams, selfv)
        parity.compare(runs[1].numpy(), ob.render(threads=16), label=f"sparse edits step {step}")
    assert total_edits > 1000


def test_sparse_edits_raise_the_top_layer_and_reject_bad_input(lib, orc):
    grid = (12, 10, 9)
    rng = np.random.default_rng(5)
    vox = np.zeros((2, 9, 10, 12), np.uint8)
    vox[:, 0] = 1                                           # floor only: highest solid layer is 0
    pal = rng.integers(0, 256, size=(2, 4, 3), dtype=np.uint8)
    cams = np.array([[2.5, 5.5, 1.5, 0.0, 0.5], [9.5, 5.5, 1.5, np.pi, 0.4]] * 2, np.float32)
    spec = _mini_spec(2, 2, grid, 64, 40, 3)
    run = _gpu_for(spec, vox, pal, cams)
    ob = _oracle_for(orc, spec, vox, pal, cams)
    # a floating slab high above the floor, in environment 1 only
    k, j = 7, np.arange(3, 8)
    idx = np.array([(k * 10 + jj) * 12 + ii for jj in j for ii in range(4, 9)], np.int32)
    env = np.ones_like(idx)
    mat = np.full(idx.shape, 3, np.uint8)
    run.batch.update_voxels(env, idx, mat)
    ob.update_voxels(env, idx, mat)
    run.render()
    g, ref = run.numpy(), ob.render()
    parity.compare(g, ref, label="slab added by edits")
    assert (g.material[2:] == 3).any() and not (g.material[:2] == 3).any()
    # remove it again: back to the floor-only picture
    run.batch.update_voxels(env, idx, np.zeros_like(mat))
    ob.update_voxels(env, idx, np.zeros_like(mat))
    run.render()
    parity.compare(run.numpy(), ob.render(), label="slab removed by edits")
    assert not (run.numpy().material == 3).any()
    for bad in ((np.array([2], np.int32), np.array([0], np.int32), np.array([1], np.uint8)),
                (np.array([0], np.int32), np.array([12 * 10 * 9], np.int32), np.array([1], np.uint8)),
                (np.array([0], np.int32), np.array([5], np.int32), np.array([4], np.uint8))):
        with pytest.raises(binding.MvError) as e:
            run.batch.update_voxels(*bad)
        assert e.value.code == binding.MV_ERR_RANGE
    run.batch.update_voxels(np.zeros(0, np.int32), np.zeros(0, np.int32), np.zeros(0, np.uint8))      # empty: no-op
    # device-side edits out of range are dropped, not applied
    run.batch.update_voxels(torch.tensor([5, 0], dtype=torch.int32).cuda(), torch.tensor([0, 10 ** 6], dtype=torch.int32).cuda(),
                            torch.tensor([1, 1], dtype=torch.uint8).cuda(), stream=_stream())
    torch.cuda.synchronize()
    run.render()
    parity.compare(run.numpy(), ob.render(), label="after dropped edits")


# ------------------------------------------------------------------------------------------ config 4
def test_config4_large_grid_large_image(lib, orc):
    wl = synth.generate(4)
    spec = wl.spec
    run = _gpu_for(spec, wl.voxels, wl.palette, wl.cameras[0])
    run.render()
    ob = _oracle_for(orc, spec, wl.voxels, wl.palette, wl.cameras[0])
    total = _compare_all(ob, run, "cfg4", chunk=128)
    assert total["pixels"] == spec.num_obs * spec.width * spec.height
    plain = GpuRender(run.batch, spec.width, spec.height, aux=False)
    plain.render()
    assert torch.equal(plain.rgb, run.rgb) and torch.equal(plain.depth.view(torch.int32), run.depth.view(torch.int32))


# ------------------------------------------------------------------------------------------ edge cases
def _mini_spec(N, A, grid, W, H, M):
    return synth.WorkloadSpec("mini", -1, N, A, grid, W, H, M, 1)


@pytest.mark.parametrize("grid,W,H", [((7, 5, 3), 33, 19), ((1, 1, 1), 1, 1), ((8, 8, 4), 2, 2), ((5, 9, 2), 30, 17),
                                      ((40, 40, 16), 130, 70), ((33, 2, 31), 64, 8), ((70, 9, 5), 40, 24),
                                      ((64, 64, 6), 48, 32), ((9, 100, 4), 36, 20), ((63, 64, 3), 40, 24),
                                      ((64, 1, 2), 16, 16), ((1, 64, 2), 24, 8), ((17, 63, 9), 128, 72),
                                      ((64, 64, 40), 64, 40), ((64, 64, 75), 32, 24)])
def test_unstructured_worlds_odd_sizes_cameras_anywhere(lib, orc, grid, W, H):
    """Random occupancy (overhangs, no floor), cameras inside, outside and inside solids, image sizes
    that are not multiples of the tile or of four, grids whose voxel count is not a multiple of 32."""
    rng = np.random.default_rng(hash((grid, W, H)) % (2 ** 31))
    N, A, M = 5, 3, 255
    spec = _mini_spec(N, A, grid, W, H, M)
    for fill in (0.0, 0.1, 0.5, 1.0):
        vox, pal = synth.random_world(rng, N, grid, fill, M)
        cams = synth.random_cameras(rng, N * A, grid, margin=2.0)
        ob = _oracle_for(orc, spec, vox, pal, cams)
        ref = ob.render()
        for device_src in (True, False):
            run = _gpu_for(spec, vox, pal, cams, device_src=device_src)
            run.render()
            g = run.numpy()
            # tiny images cannot meet a per-image percentage; judge them on admissibility alone
            differ = (g.hit_index != ref.hit_index) | (g.material != ref.material) | (g.face != ref.face)
            assert not (differ & ~(ref.edge_margin < parity.EDGE_MARGIN)).any()
            same = ~differ
            assert (np.abs(g.rgb.astype(int) - ref.rgb.astype(int)).max(axis=-1)[same] <= 1).all()
            np.testing.assert_allclose(g.depth[same], ref.depth[same], rtol=1e-4, atol=0)
            assert differ.mean() <= 0.002


@pytest.mark.parametrize("hfov", [0.2, 1.0, 2.6, 3.0])
def test_narrow_and_wide_fields_of_view(lib, orc, hfov):
    """Horizontal fields of view from 11 to 172 degrees on an arena world: parity at every pixel."""
    wl = synth.generate(1, num_envs=6)
    spec = wl.spec
    ob = _oracle_for(orc, spec, wl.voxels, wl.palette, wl.cameras[0], hfov_rad=hfov)
    run = _gpu_for(spec, wl.voxels, wl.palette, wl.cameras[0], hfov_rad=hfov)
    run.render()
    parity.compare(run.numpy(), ob.render(threads=8), label=f"hfov {hfov}")


def test_cameras_exactly_on_voxel_planes(lib, orc):
    """Cameras whose x, y or z is an integer sit on a voxel plane: the cell is floor(P), and a solid
    neighbour across the plane is hit at depth 0 through that plane's face.  One integer coordinate is not
    a tie (the margin looks at the other two axes), so these pixels must match exactly."""
    grid = (9, 7, 5)
    rng = np.random.default_rng(77)
    N, A, M = 6, 6, 9
    spec = _mini_spec(N, A, grid, 40, 24, M)
    vox, pal = synth.random_world(rng, N, grid, 0.35, M)
    cams = synth.random_cameras(rng, N * A, grid, margin=0.0)
    cams[:, 0] = np.clip(cams[:, 0], 0.2, grid[0] - 0.2)
    cams[:, 1] = np.clip(cams[:, 1], 0.2, grid[1] - 0.2)
    cams[:, 2] = np.clip(cams[:, 2], 0.2, grid[2] - 0.2)
    for o in range(N * A):
        axis = o % 3
        # on an interior plane of that axis, or (every fourth camera) on the grid boundary itself
        cams[o, axis] = float(rng.integers(1, grid[axis])) if o % 4 else float(rng.choice([0, grid[axis]]))
    ob = _oracle_for(orc, spec, vox, pal, cams)
    ref = ob.render()
    run = _gpu_for(spec, vox, pal, cams)
    run.render()
    g = run.numpy()
    differ = (g.hit_index != ref.hit_index) | (g.material != ref.material) | (g.face != ref.face)
    assert not (differ & ~(ref.edge_margin < parity.EDGE_MARGIN)).any()
    same = ~differ
    assert (np.abs(g.rgb.astype(int) - ref.rgb.astype(int)).max(axis=-1)[same] <= 1).all()
    np.testing.assert_allclose(g.depth[same], ref.depth[same], rtol=1e-4, atol=0)
    assert ((ref.depth == 0) & (ref.hit_index >= 0) & (ref.face < 6)).any(), "some pixel hits a neighbour at depth 0"


def _random_configuration(seed):
    """One odd but valid configuration: grid and image sizes, occupancy, cameras snapped to cell centres, to
    voxel planes, to grid corners or left anywhere (also outside), special yaw and pitch values, a random
    field of view, sometimes own bodies."""
    rng = np.random.default_rng(seed)
    wide = rng.random() < 0.1
    grid = (int(rng.integers(1, 130 if wide else 65)), int(rng.integers(1, 65)), int(rng.integers(1, 21)))
    W, H = int(rng.integers(1, 71)), int(rng.integers(1, 41))
    if rng.random() < 0.4:
        W, H = 8 * int(rng.integers(1, 9)), 8 * int(rng.integers(1, 5))
    N, A, M = 3, 2, int(rng.integers(1, 256))
    vox, pal = synth.random_world(rng, N, grid, float(rng.choice([0.0, 0.03, 0.2, 0.6, 1.0])), M)
    if rng.random() < 0.5:
        vox[:, 0] = np.maximum(vox[:, 0], 1)                       # a floor
    cams = synth.random_cameras(rng, N * A, grid, margin=float(rng.choice([0.0, 0.0, 1.5])))
    for o in range(N * A):
        mode = rng.integers(0, 6)
        if mode == 0:
            for a in range(3):
                cams[o, a] = np.floor(np.clip(cams[o, a], 0, grid[a] - 1)) + 0.5
        elif mode == 1:
            a = int(rng.integers(0, 3))
            cams[o, a] = float(rng.integers(0, grid[a] + 1))
        elif mode == 2:
            for a in range(3):
                cams[o, a] = float(rng.integers(0, grid[a] + 1))
        if rng.random() < 0.3:
            cams[o, 3] = float(rng.integers(0, 8)) * np.float32(np.pi / 4)
        if rng.random() < 0.2:
            cams[o, 4] = float(rng.choice([0.0, np.pi / 2, -np.pi / 2, np.pi / 4]))
    selfv = rng.integers(-1, grid[0] * grid[1] * grid[2], size=N * A).astype(np.int32) if rng.random() < 0.4 else None
    hfov = float(np.float32(rng.choice([np.pi / 2, rng.uniform(0.05, 3.1)])))
    return grid, W, H, N, A, M, vox, pal, cams.astype(np.float32), selfv, hfov


def test_randomized_configurations_against_the_oracle(lib, orc):
    """1500 small random configurations (see _random_configuration): every pixel must satisfy the parity rule.
    Small images cannot meet a per-image percentage of exact pixels (a camera on a voxel plane makes most of
    its pixels ties), so the rule is applied pixel by pixel: a difference in hit, material or face needs an
    edge margin below the threshold; everywhere else colour within 1 LSB and depth within 1e-4 relative.
    (This sweep found the two cases that the structured workloads never reach: a camera a few 1e-3 voxels
    in front of a wall, and a camera exactly on a voxel plane.)"""
    pixels = 0
    for seed in range(7000, 8500):
        grid, W, H, N, A, M, vox, pal, cams, selfv, hfov = _random_configuration(seed)
        ob = orc.OracleBatch(N, A, grid, W, H, M, hfov_rad=hfov)
        ob.upload_worlds(vox, pal)
        ob.set_cameras(cams, selfv)
        ref = ob.render()
        batch = binding.Batch(N, A, grid, M, W, H, hfov_rad=hfov)
        batch.upload_worlds(torch.from_numpy(vox).cuda(), torch.from_numpy(pal).cuda(), stream=_stream())
        batch.set_cameras(torch.from_numpy(cams).cuda(), None if selfv is None else torch.from_numpy(selfv).cuda(),
                          stream=_stream())
        run = GpuRender(batch, W, H, aux=True)
        run.render()
        g = run.numpy()
        _pixelwise_rule(g, ref, f"seed {seed} grid {grid} image {W}x{H}")
        pixels += g.depth.size
        batch.close()
        ob.close()
    assert pixels > 5_000_000


def _pixelwise_rule(g, ref, where):
    differ = (g.hit_index != ref.hit_index) | (g.material != ref.material) | (g.face != ref.face)
    assert not (differ & ~(ref.edge_margin < parity.EDGE_MARGIN)).any(), where
    same = ~differ
    assert (np.abs(g.rgb.astype(int) - ref.rgb.astype(int)).max(axis=-1)[same] <= 1).all(), where
    assert (np.abs(g.depth - ref.depth)[same] <= 1e-4 * np.abs(ref.depth)[same]).all(), where


def test_randomized_entry_point_sequences(lib, orc):
    """300 random configurations driven through the other entry points: per-environment uploads in random
    order from host or device memory, a random launch shape, the colour+depth-only launch against the one
    with auxiliary outputs (bit for bit), random sparse edits (sets and clears) from host or device memory,
    a random active mask, and a random indicator bar -- each step against the oracle."""
    for seed in range(9000, 9300):
        grid, W, H, N, A, M, vox, pal, cams, selfv, hfov = _random_configuration(seed)
        rng = np.random.default_rng(seed + 10 ** 6)
        X, Y, Z = grid
        where = f"seed {seed} grid {grid} image {W}x{H}"
        ob = orc.OracleBatch(N, A, grid, W, H, M, hfov_rad=hfov)
        batch = binding.Batch(N, A, grid, M, W, H, hfov_rad=hfov, tiles_per_block=int(rng.choice([0, 1, 2, 3, 5, 8, 1000])))
        for e in rng.permutation(N):
            v, p_ = vox[e:e + 1], pal[e:e + 1]
            if rng.random() < 0.5:
                batch.upload_worlds(torch.from_numpy(v).cuda(), torch.from_numpy(p_).cuda(), first_env=int(e), stream=_stream())
            else:
                batch.upload_worlds(v, p_, first_env=int(e), stream=_stream())
        torch.cuda.synchronize()
        ob.upload_worlds(vox, pal)
        batch.set_cameras(torch.from_numpy(cams).cuda(), None if selfv is None else torch.from_numpy(selfv).cuda(),
                          stream=_stream())
        ob.set_cameras(cams, selfv)
        full = GpuRender(batch, W, H, aux=True)
        full.render()
        _pixelwise_rule(full.numpy(), ob.render(), where + " uploads")
        plain = GpuRender(batch, W, H, aux=False)
        plain.render()
        assert torch.equal(plain.rgb, full.rgb) and torch.equal(plain.depth.view(torch.int32), full.depth.view(torch.int32)), where
        # sparse edits, each voxel at most once
        flat = rng.choice(N * X * Y * Z, size=min(int(rng.integers(1, 200)), N * X * Y * Z), replace=False)
        env, idx = (flat // (X * Y * Z)).astype(np.int32), (flat % (X * Y * Z)).astype(np.int32)
        mat = np.where(rng.random(env.size) < 0.5, 0, rng.integers(1, M + 1, size=env.size)).astype(np.uint8)
        if rng.random() < 0.5:
            batch.update_voxels(torch.from_numpy(env).cuda(), torch.from_numpy(idx).cuda(), torch.from_numpy(mat).cuda(),
                                stream=_stream())
        else:
            batch.update_voxels(env, idx, mat, stream=_stream())
        torch.cuda.synchronize()
        ob.update_voxels(env, idx, mat)
        full.render()
        ref = ob.render()
        _pixelwise_rule(full.numpy(), ref, where + " edits")
        # active mask and bar
        active = (rng.random(N) < 0.6).astype(np.uint8)
        batch.set_active(torch.from_numpy(active).cuda() if rng.random() < 0.5 else active, stream=_stream())
        rendered = full.rgb.cpu().numpy()
        full.rgb.fill_(9); full.depth.fill_(-3.0)
        batch.render(full.rgb, full.depth, full.material, full.hit, full.face, stream=_stream())
        bw, bh = int(rng.integers(1, W + 1)), int(rng.integers(1, H + 1))
        bx, by = int(rng.integers(0, W - bw + 1)), int(rng.integers(0, H - bh + 1))
        frac = rng.uniform(-0.2, 1.2, size=N * A).astype(np.float32)
        batch.draw_bars(full.rgb, torch.from_numpy(frac).cuda() if rng.random() < 0.5 else frac, bx, by, bw, bh,
                        (255, 0, 0), (10, 20, 30), stream=_stream())
        torch.cuda.synchronize()
        want = ref.rgb.copy()
        ob.draw_bars(want, frac, bx, by, bw, bh, (255, 0, 0), (10, 20, 30), active=active)
        got, got_d = full.rgb.cpu().numpy(), full.depth.cpu().numpy()
        on = np.repeat(active.astype(bool), A)
        inside = np.zeros((H, W), bool)
        inside[by:by + bh, bx:bx + bw] = True
        assert (got[~on] == 9).all() and (got_d[~on] == -3.0).all(), where + ": inactive environments were touched"
        assert (got[on][:, inside] == want[on][:, inside]).all(), where + ": bar pixels"
        assert (got[on][:, ~inside] == rendered[on][:, ~inside]).all(), where + ": pixels outside the bar"
        batch.close()
        ob.close()


def test_randomized_reupload_sequences(lib, orc):
    """200 random configurations, five rounds each on one batch: new worlds that are lower, taller, empty in one
    environment or have a layer of air in the middle, uploaded from device memory (copied), from host memory, borrowed
    from a device array, or for a range of environments only; palettes replaced or kept; new cameras; every round
    against the oracle.  (Layers of air are neither copied nor packed through LDS: stale material bytes stay behind
    zero rows, and the staged layers follow the tallest world heard of.)"""
    for seed in range(12000, 12200):
        grid, W, H, N, A, M, vox, pal, cams, selfv, hfov = _random_configuration(seed)
        rng = np.random.default_rng(seed + 7 * 10 ** 6)
        X, Y, Z = grid
        ob = orc.OracleBatch(N, A, grid, W, H, M, hfov_rad=hfov)
        batch = binding.Batch(N, A, grid, M, W, H, hfov_rad=hfov)
        run = GpuRender(batch, W, H, aux=True)
        borrowed = []                                   # device arrays the batch may still read
        cur_v, cur_p = vox.copy(), pal.copy()
        for rnd in range(5):
            first = rnd == 0
            if first:
                v2, p2 = cur_v, cur_p
            else:
                v2, p2 = synth.random_world(rng, N, grid, float(rng.choice([0.0, 0.05, 0.3, 0.8])), M)
                v2[:, int(rng.integers(0, Z + 1)):] = 0
                if rng.random() < 0.3:
                    v2[int(rng.integers(0, N))] = 0
                if rng.random() < 0.3 and Z > 2:
                    v2[:, int(rng.integers(1, Z))] = 0
            mode = int(rng.integers(0, 3 if first else 4))
            new_pal = first or rng.random() < 0.5
            where = f"seed {seed} round {rnd} mode {mode} grid {grid} image {W}x{H}"
            if mode == 0:
                batch.upload_worlds(torch.from_numpy(v2).cuda(), torch.from_numpy(p2).cuda() if new_pal else None, stream=_stream())
            elif mode == 1:
                batch.upload_worlds(v2, p2 if new_pal else None, stream=_stream())
            elif mode == 2:
                borrowed.append(torch.from_numpy(v2).cuda())
                batch.upload_worlds(borrowed[-1], torch.from_numpy(p2).cuda() if new_pal else None, stream=_stream(), borrow=True)
            else:
                # a range of environments: the batch must own its grids for that, so a borrowing ends first
                batch.upload_worlds(torch.from_numpy(cur_v).cuda(), None, stream=_stream())
                e0 = int(rng.integers(0, N))
                cnt = int(rng.integers(1, N - e0 + 1))
                src, psrc = np.ascontiguousarray(v2[e0:e0 + cnt]), np.ascontiguousarray(p2[e0:e0 + cnt])
                if rng.random() < 0.5:
                    batch.upload_worlds(torch.from_numpy(src).cuda(), torch.from_numpy(psrc).cuda() if new_pal else None,
                                        first_env=e0, stream=_stream())
                else:
                    batch.upload_worlds(src, psrc if new_pal else None, first_env=e0, stream=_stream())
                v2 = cur_v.copy()
                v2[e0:e0 + cnt] = src
                if new_pal:
                    p2, keep = cur_p.copy(), p2
                    p2[e0:e0 + cnt] = keep[e0:e0 + cnt]
            cur_v = v2
            if new_pal:
                cur_p = p2
            ob.upload_worlds(cur_v, cur_p)
            c2 = synth.random_cameras(rng, N * A, grid, margin=float(rng.choice([0.0, 0.5])))
            batch.set_cameras(torch.from_numpy(c2).cuda(), stream=_stream())
            ob.set_cameras(c2)
            torch.cuda.synchronize()
            run.render()
            _pixelwise_rule(run.numpy(), ob.render(), where)
        batch.close()
        ob.close()


def test_worlds_taller_than_the_staged_layers(lib, orc):
    """The render keeps only the lowest layers of a grid on chip (as many as the tallest world it has heard of
    needs).  With that number forced below what the worlds need, every workgroup traces through device
    memory instead: same parity rule, own bodies still invisible.  Back on the automatic choice, the second
    render after a synchronisation (which has learnt the height from the upload) equals the first bit for bit."""
    wl = synth.generate(3, num_envs=12)
    spec = wl.spec
    ob = _oracle_for(orc, spec, wl.voxels, wl.palette, wl.cameras[0], wl.self_voxel[0])
    ref = ob.render(threads=8)
    run = _gpu_for(spec, wl.voxels, wl.palette, wl.cameras[0], wl.self_voxel[0])
    run.render()                                   # before any feedback: all layers staged
    first = run.numpy()
    parity.compare(first, ref, label="all layers staged")
    torch.cuda.synchronize()
    run.render()                                   # now with as many layers as the worlds need
    second = run.numpy()
    for name in ("rgb", "depth", "material", "hit_index", "face"):
        np.testing.assert_array_equal(getattr(second, name).view(np.uint8), getattr(first, name).view(np.uint8))
    for layers in (1, 2, 5):
        run.batch.debug_set_staged_layers(layers)
        run.render()
        parity.compare(run.numpy(), ref, label=f"{layers} layers staged")
    run.batch.debug_set_staged_layers(spec.grid[2])
    run.render()
    forced_all = run.numpy()
    for name in ("rgb", "depth", "material", "hit_index", "face"):
        np.testing.assert_array_equal(getattr(forced_all, name).view(np.uint8), getattr(first, name).view(np.uint8))
    with pytest.raises(binding.MvError):
        run.batch.debug_set_staged_layers(spec.grid[2] + 1)
    run.batch.debug_set_staged_layers(0)


def test_cameras_above_every_solid(lib, orc):
    """Cameras that fly above their world (the row scan treats everything from the top of the solids upwards
    as one tall empty layer), looking down, level and up, over worlds of different heights in one batch."""
    grid = (24, 20, 12)
    rng = np.random.default_rng(5)
    N, A, M = 6, 4, 7
    spec = _mini_spec(N, A, grid, 64, 40, M)
    vox, pal = synth.random_world(rng, N, grid, 0.25, M)
    for n in range(N):
        vox[n, 2 + n:] = 0                          # world n is 2 + n layers tall
    vox[N - 1] = 0                                  # and one empty world
    cams = synth.random_cameras(rng, N * A, grid, margin=0.0, max_pitch=1.4)
    for o in range(N * A):
        n = o // A
        cams[o, 2] = rng.uniform(2 + n, grid[2]) if o % A else float(2 + n)     # above the top; agent 0 exactly on it
    cams = cams.astype(np.float32)
    ob = _oracle_for(orc, spec, vox, pal, cams)
    ref = ob.render()
    run = _gpu_for(spec, vox, pal, cams)
    for _ in range(2):                              # all layers staged, then as many as the tallest world needs
        run.render()
        _pixelwise_rule(run.numpy(), ref, "flying cameras")
        torch.cuda.synchronize()
    assert (ref.hit_index >= 0).mean() > 0.2


def test_axis_parallel_and_vertical_rays(lib, orc):
    grid = (6, 6, 6)
    vox = np.zeros((1, 6, 6, 6), np.uint8)
    vox[0, 0] = 1
    vox[0, 5, 2, 2] = 2
    vox[0, 2, 2, 5] = 1
    pal = np.full((1, 3, 3), 200, np.uint8)
    cams = np.array([[2.5, 2.5, 2.5, 0.0, -np.pi / 2], [2.5, 2.5, 2.5, 0.0, np.pi / 2], [0.5, 2.5, 2.5, 0.0, 0.0],
                     [0.5, 3.5, 2.5, 0.0, 0.0]], np.float32)
    for (W, H, hfov) in ((1, 1, float(np.float32(np.pi / 2))), (2, 2, 1e-3)):
        spec = _mini_spec(1, 4, grid, W, H, 2)
        ob = _oracle_for(orc, spec, vox, pal, cams, hfov_rad=hfov)
        run = _gpu_for(spec, vox, pal, cams, hfov_rad=hfov)
        run.render()
        g, ref = run.numpy(), ob.render()
        np.testing.assert_array_equal(g.hit_index, ref.hit_index)
        np.testing.assert_array_equal(g.face, ref.face)
        np.testing.assert_allclose(g.depth, ref.depth, rtol=1e-6)
        np.testing.assert_array_equal(g.rgb, ref.rgb)


def test_custom_light_sky_and_fov(lib, orc):
    wl = synth.generate(0)
    kw = dict(hfov_rad=1.0, light_dir=(-3.0, 0.5, 1.0), ambient=0.15, diffuse=0.95, sky_rgb=(1, 2, 3))
    ob = _oracle_for(orc, wl.spec, wl.voxels, wl.palette, wl.cameras[0], **kw)
    run = _gpu_for(wl.spec, wl.voxels, wl.palette, wl.cameras[0], **kw)
    run.render()
    st = parity.compare(run.numpy(), ob.render(), sky_rgb=(1, 2, 3), label="custom light")
    assert st["colour_exact_fraction"] == 1.0


def test_partial_uploads_and_palette_keep(lib, orc):
    wl = synth.generate(1, num_envs=8)
    spec = wl.spec
    ob = _oracle_for(orc, spec, wl.voxels, wl.palette, wl.cameras[0])
    batch = binding.Batch(spec.num_envs, spec.agents_per_env, spec.grid, spec.num_materials, spec.width, spec.height)
    run = GpuRender(batch, spec.width, spec.height)
    cams_d = torch.from_numpy(wl.cameras[0]).cuda()
    # render before anything is there
    with pytest.raises(binding.MvError) as e:
        batch.render(run.rgb, run.depth, stream=_stream())
    assert e.value.code == binding.MV_ERR_STATE
    batch.upload_worlds(wl.voxels[:3], wl.palette[:3], first_env=0)
    batch.set_cameras(cams_d, stream=_stream())
    with pytest.raises(binding.MvError) as e:
        batch.render(run.rgb, run.depth, stream=_stream())
    assert e.value.code == binding.MV_ERR_STATE
    batch.upload_worlds(torch.from_numpy(wl.voxels[3:]).cuda(), torch.from_numpy(wl.palette[3:]).cuda(), first_env=3,
                        stream=_stream())
    torch.cuda.synchronize()
    run.render()
    parity.compare(run.numpy(), ob.render(threads=8), label="partial uploads")
    # replace two grids in the middle, keep their palettes
    swapped = wl.voxels.copy()
    swapped[4:6] = wl.voxels[6:8]
    batch.upload_worlds(swapped[4:6], None, first_env=4)
    ob.upload_worlds(swapped[4:6], None, first_env=4)
    run.render()
    parity.compare(run.numpy(), ob.render(threads=8), label="grid swap, palette kept")
    # range and content errors leave the batch untouched
    with pytest.raises(binding.MvError) as e:
        batch.upload_worlds(wl.voxels[:2], wl.palette[:2], first_env=7)
    assert e.value.code == binding.MV_ERR_RANGE
    bad = wl.voxels[:1].copy()
    bad[0, 3, 3, 3] = spec.num_materials + 1
    with pytest.raises(binding.MvError) as e:
        batch.upload_worlds(bad, None, first_env=0)
    assert e.value.code == binding.MV_ERR_RANGE
    bad_cams = wl.cameras[0].copy()
    bad_cams[5, 3] = np.nan
    with pytest.raises(binding.MvError) as e:
        batch.set_cameras(bad_cams)
    assert e.value.code == binding.MV_ERR_ARG
    run.render()
    parity.compare(run.numpy(), ob.render(threads=8), label="after rejected calls")


@pytest.mark.parametrize("grid", [(63, 9, 4), (64, 9, 4), (9, 63, 4), (9, 64, 4), (62, 63, 3), (40, 40, 5)])
def test_rays_that_reach_the_far_end_of_a_row(lib, orc, grid):
    """Rows of 63 cells and fewer are scanned without clamping the last cell of a run, rows of 64 cells
    with the clamp: rays that run the whole length of a row, towards either end, with solids in the last
    column, next to it, or nowhere, and cameras close to or on the near and far boundary."""
    X, Y, Z = grid
    rng = np.random.default_rng(X * 1000 + Y)
    N, A, M = 6, 4, 5
    spec = _mini_spec(N, A, grid, 48, 16, M)
    vox = np.zeros((N, Z, Y, X), np.uint8)
    for e in range(N):
        if e % 3 == 0:                       # solids in the outermost columns only, at random rows and layers
            for col in (0, X - 1):
                vox[e, :, :, col] = np.where(rng.random((Z, Y)) < 0.5, rng.integers(1, M + 1, (Z, Y)), 0)
            for row in (0, Y - 1):
                vox[e, :, row, :] = np.where(rng.random((Z, X)) < 0.5, rng.integers(1, M + 1, (Z, X)), 0)
        elif e % 3 == 1:                     # the column next to the outermost one
            vox[e, :, :, X - 2] = rng.integers(0, M + 1, (Z, Y))
            vox[e, :, :, 1] = rng.integers(0, M + 1, (Z, Y))
            vox[e, :, Y - 2, :] = rng.integers(0, M + 1, (Z, X))
        # e % 3 == 2: empty world, every ray leaves through the far side
    pal = rng.integers(0, 256, (N, M + 1, 3)).astype(np.uint8)
    cams = np.zeros((N * A, 5), np.float32)
    for o in range(N * A):
        towards = o % 4                      # +x, -x, +y, -y, each nearly parallel to the rows
        yaw = (0.0, np.pi, np.pi / 2, -np.pi / 2)[towards] + rng.uniform(-0.02, 0.02)
        near = rng.choice([0.0, 1e-3, 0.5, 1.0])
        pos = [rng.uniform(0.1, X - 0.1), rng.uniform(0.1, Y - 0.1), rng.uniform(0.1, Z - 0.1)]
        if towards == 0: pos[0] = near
        if towards == 1: pos[0] = X - near
        if towards == 2: pos[1] = near
        if towards == 3: pos[1] = Y - near
        cams[o] = (pos[0], pos[1], pos[2], yaw, rng.uniform(-0.02, 0.02))
    hfov = 0.3
    ob = _oracle_for(orc, spec, vox, pal, cams, hfov_rad=hfov)
    run = _gpu_for(spec, vox, pal, cams, hfov_rad=hfov)
    run.render()
    g, ref = run.numpy(), ob.render()
    _pixelwise_rule(g, ref, f"far end of rows, grid {grid}")
    assert (ref.hit_index >= 0).any() and (ref.hit_index < 0).any()


def test_largest_grid_the_lds_plan_takes(lib, orc):
    grid = (128, 128, 32)                   # 64 KiB of occupancy bits
    rng = np.random.default_rng(8)
    spec = _mini_spec(2, 2, grid, 64, 40, 9)
    vox, pal = synth.random_world(rng, 2, grid, 0.01, 9)
    vox[:, 0] = 3
    cams = synth.random_cameras(rng, 4, grid, margin=0.0, max_pitch=0.6)
    cams[:, 2] = 1.5 + cams[:, 2] % 20
    ob = _oracle_for(orc, spec, vox, pal, cams)
    run = _gpu_for(spec, vox, pal, cams)
    run.render()
    parity.compare(run.numpy(), ob.render(threads=4), label="128x128x32 grid")


@pytest.mark.parametrize("W,H", [(1920, 1080), (16384, 8), (8, 4096), (8, 16384)])
def test_largest_images(lib, orc, W, H):
    """Images far larger than the paper's 128x72, up to the largest width and height a configuration may name:
    thousands of tiles per observation, strips much shorter than an observation, pixel scalars and row records that
    fill most of a workgroup's LDS.  Either the batch is refused at creation for lack of LDS (MV_ERR_CAPACITY, nothing
    half-made) or every pixel is held to the parity rule."""
    wl = synth.generate(1, num_envs=2)
    spec = _mini_spec(2, 1, wl.spec.grid, W, H, wl.spec.num_materials)
    cams = np.ascontiguousarray(wl.cameras[0][::wl.spec.agents_per_env][:2])
    try:
        run = _gpu_for(spec, wl.voxels, wl.palette, cams)
    except binding.MvError as e:
        assert e.code == binding.MV_ERR_CAPACITY and H > 4096, (W, H, e.code, str(e))
        return
    run.render()
    ob = _oracle_for(orc, spec, wl.voxels, wl.palette, cams)
    parity.compare(run.numpy(), ob.render(threads=8), label=f"{W}x{H} image")


def test_borrowed_worlds_render_the_same_bits(lib, orc):
    """mv_upload_worlds with MV_SRC_DEVICE_BORROWED: no material copy, the render reads the caller's device array.
    The images equal those of a copying upload bit for bit; changing the array and uploading again re-packs; edits and
    partial uploads are refused while the batch borrows, and a copying upload of all environments ends that."""
    wl = synth.generate(3, num_envs=48)
    spec = wl.spec
    cams, selfv = wl.cameras[0], wl.self_voxel[0]
    copied = _gpu_for(spec, wl.voxels, wl.palette, cams, self_voxel=selfv)
    copied.render()
    want = copied.numpy()
    parity.compare(want, _oracle_for(orc, spec, wl.voxels, wl.palette, cams, selfv).render(threads=8), label="copied upload")
    batch = binding.Batch(spec.num_envs, spec.agents_per_env, spec.grid, spec.num_materials, spec.width, spec.height)
    own = torch.from_numpy(wl.voxels).cuda()                   # the simulator's own array
    pal = torch.from_numpy(wl.palette).cuda()
    batch.upload_worlds(own, pal, stream=_stream(), borrow=True)
    batch.set_cameras(torch.from_numpy(cams).cuda(), torch.from_numpy(selfv).cuda(), stream=_stream())
    run = GpuRender(batch, spec.width, spec.height, aux=True)
    run.render()
    g = run.numpy()
    for name in ("rgb", "material", "hit_index", "face"):
        np.testing.assert_array_equal(getattr(g, name), getattr(want, name), err_msg=name)
    np.testing.assert_array_equal(g.depth.view(np.uint32), want.depth.view(np.uint32))
    # refused while borrowing
    one = torch.zeros(1, dtype=torch.int32, device="cuda")
    for call in (lambda: batch.update_voxels(one, one, torch.ones(1, dtype=torch.uint8, device="cuda")),
                 lambda: batch.move_voxels(one, one, one + 1, torch.ones(1, dtype=torch.uint8, device="cuda")),
                 lambda: batch.upload_worlds(own[:4], pal[:4], first_env=0, count=4, stream=_stream())):
        with pytest.raises(binding.MvError) as e:
            call()
        assert e.value.code == binding.MV_ERR_STATE
    with pytest.raises(binding.MvError) as e:
        batch.upload_worlds(own[:4], pal[:4], first_env=0, count=4, stream=_stream(), borrow=True)
    assert e.value.code == binding.MV_ERR_ARG
    # the simulator moves on: the next step's worlds written into the same array, packed again without a copy
    vox2, cams2, selfv2 = synth.dynamic_step(wl)
    own.copy_(torch.from_numpy(vox2).cuda())
    batch.upload_worlds(own, None, stream=_stream(), borrow=True)
    batch.set_cameras(torch.from_numpy(cams2).cuda(), torch.from_numpy(selfv2).cuda(), stream=_stream())
    run.render()
    parity.compare(run.numpy(), _oracle_for(orc, spec, vox2, wl.palette, cams2, selfv2).render(threads=8), label="borrowed, next step")
    # a copying upload ends the borrowing: the caller's array may change or go away
    batch.upload_worlds(own, None, stream=_stream())
    torch.cuda.synchronize()
    own.zero_()
    torch.cuda.synchronize()
    run.render()
    parity.compare(run.numpy(), _oracle_for(orc, spec, vox2, wl.palette, cams2, selfv2).render(threads=8), label="copied again")
    batch.update_voxels(one, one, torch.ones(1, dtype=torch.uint8, device="cuda"))      # edits work again


def test_fetch_observations_into_pinned_and_pageable_memory(lib):
    """The device-to-host copy of a range of observations equals what the device tensors hold, for pinned
    memory from the library and for ordinary NumPy arrays, and rejects ranges outside the batch."""
    wl = synth.generate(1, num_envs=8)
    spec = wl.spec
    run = _gpu_for(spec, wl.voxels, wl.palette, wl.cameras[0], aux=False)
    run.render()
    H, W = spec.height, spec.width
    first, count = 5, 19
    pin_rgb = binding.PinnedBuffer(count * H * W * 3)
    pin_depth = binding.PinnedBuffer(count * H * W * 4)
    try:
        run.batch.fetch_observations(run.rgb, run.depth, first, count, pin_rgb.address, pin_depth.address, stream=_stream())
        page_rgb = np.zeros((count, H, W, 3), np.uint8)
        run.batch.fetch_observations(run.rgb, None, first, count, page_rgb, None, stream=_stream())
        torch.cuda.synchronize()
        want_rgb = run.rgb[first:first + count].cpu().numpy()
        want_depth = run.depth[first:first + count].cpu().numpy()
        assert np.array_equal(pin_rgb.array(np.uint8, (count, H, W, 3)), want_rgb)
        assert np.array_equal(pin_depth.array(np.float32, (count, H, W)).view(np.uint32), want_depth.view(np.uint32))
        assert np.array_equal(page_rgb, want_rgb)
        with pytest.raises(binding.MvError):
            run.batch.fetch_observations(run.rgb, run.depth, spec.num_obs - 3, 4, pin_rgb.address, None, stream=_stream())
        with pytest.raises(binding.MvError):
            run.batch.fetch_observations(None, run.depth, 0, 1, pin_rgb.address, None, stream=_stream())
    finally:
        torch.cuda.synchronize()
        pin_rgb.close(); pin_depth.close()


def test_active_mask_and_indicator_bars(lib, orc):
    """Inactive environments are neither rendered nor painted (their pixels keep what the caller's
    tensors held); active ones are bit for bit what a full render gives; bars match the oracle."""
    wl = synth.generate(1, num_envs=24)
    spec = wl.spec
    rng = np.random.default_rng(31)
    ob = _oracle_for(orc, spec, wl.voxels, wl.palette, wl.cameras[0])
    ref = ob.render(threads=8)
    run = _gpu_for(spec, wl.voxels, wl.palette, wl.cameras[0])
    run.render()
    full = run.numpy()
    active = (rng.random(spec.num_envs) < 0.6).astype(np.uint8)
    active[0], active[1] = 0, 1
    fractions = rng.uniform(-0.2, 1.2, size=spec.num_obs).astype(np.float32)
    fractions[:4] = [0.0, 1.0, 0.5, 0.25]
    bar = dict(x=8, y=4, width=100, height=3, fill_rgb=(255, 255, 0), empty_rgb=(40, 40, 40))
    want_rgb = ref.rgb.copy()
    ob.draw_bars(want_rgb, fractions, active=active, **bar)
    obs_active = np.repeat(active.astype(bool), spec.agents_per_env)
    for src in ("device", "host"):
        run.batch.set_active(torch.from_numpy(active).cuda() if src == "device" else active, stream=_stream())
        run.render()                                          # poisons the outputs first
        run.batch.draw_bars(run.rgb, torch.from_numpy(fractions).cuda() if src == "device" else fractions,
                            stream=_stream(), **bar)
        torch.cuda.synchronize()
        g = run.numpy()
        assert (g.rgb[~obs_active] == 7).all() and (g.depth[~obs_active] == -1.0).all() and (g.hit_index[~obs_active] == -7).all()
        np.testing.assert_array_equal(g.depth[obs_active].view(np.uint32), full.depth[obs_active].view(np.uint32))
        np.testing.assert_array_equal(g.hit_index[obs_active], full.hit_index[obs_active])
        # colours: identical to the full render outside the bar, identical to the oracle's bar inside it
        inside = np.zeros(g.rgb.shape[:3], bool)
        inside[:, 4:7, 8:108] = True
        outside = obs_active[:, None, None] & ~inside
        np.testing.assert_array_equal(g.rgb[outside], full.rgb[outside])
        np.testing.assert_array_equal(g.rgb[obs_active][:, 4:7, 8:108], want_rgb[obs_active][:, 4:7, 8:108])
    # back to all environments
    run.batch.set_active(None)
    run.render()
    parity.compare(run.numpy(), ref, label="all active again")
    with pytest.raises(binding.MvError) as e:
        run.batch.draw_bars(run.rgb, fractions, 100, 4, 100, 3, (0, 0, 0), (0, 0, 0))
    assert e.value.code == binding.MV_ERR_ARG
    bad = fractions.copy()
    bad[3] = np.inf
    with pytest.raises(binding.MvError) as e:
        run.batch.draw_bars(run.rgb, bad, 8, 4, 100, 3, (0, 0, 0), (0, 0, 0))
    assert e.value.code == binding.MV_ERR_ARG


def test_overlay_of_primitives_equals_the_oracle(lib, orc):
    """mv_draw_overlay against the oracle's overlay, byte for byte over the whole colour tensor: random lists of
    solid rectangles and gauges that overlap, values from the device and from the host, inactive environments left
    alone; the depth is not touched; one rightward gauge is the indicator bar; bad lists are refused."""
    wl = synth.generate(1, num_envs=16)
    spec = wl.spec
    W, H = spec.width, spec.height
    rng = np.random.default_rng(4711)
    ob = _oracle_for(orc, spec, wl.voxels, wl.palette, wl.cameras[0])
    run = _gpu_for(spec, wl.voxels, wl.palette, wl.cameras[0])
    active = (rng.random(spec.num_envs) < 0.7).astype(np.uint8)
    active[0], active[1] = 0, 1
    obs_active = np.repeat(active.astype(bool), spec.agents_per_env)

    def random_list(n, per_obs):
        rects = []
        for _ in range(n):
            w, h = int(rng.integers(1, W + 1)), int(rng.integers(1, H + 1))
            if rng.random() < 0.5:
                w, h = min(w, 24), min(h, 10)
            x, y = int(rng.integers(0, W - w + 1)), int(rng.integers(0, H - h + 1))
            kind = int(rng.integers(0, 3)) if per_obs > 0 else 0
            rects.append((x, y, w, h, tuple(int(v) for v in rng.integers(0, 256, 3)), kind,
                          tuple(int(v) for v in rng.integers(0, 256, 3)), int(rng.integers(0, max(per_obs, 1)))))
        return rects

    cases = [(1, 0), (1, 1), (5, 3), (12, 8), (32, 2), (7, 0)]
    for case, (n, per_obs) in enumerate(cases):
        rects = random_list(n, per_obs)
        values = None
        if per_obs > 0:
            values = rng.uniform(-0.3, 1.3, size=(spec.num_obs, per_obs)).astype(np.float32)
            values[:4, 0] = [0.0, 1.0, 0.5, 0.25]
        for src in ("device", "host"):
            run.batch.set_active(active if case % 2 == 0 else None, stream=_stream())
            run.render()                                      # poisons the outputs first
            before = run.numpy()
            given = None if values is None else (torch.from_numpy(values).cuda() if src == "device" else values)
            run.batch.draw_overlay(run.rgb, rects, given, stream=_stream())
            torch.cuda.synchronize()
            g = run.numpy()
            want = before.rgb.copy()
            ob.draw_overlay(want, rects, values, active=active if case % 2 == 0 else None)
            np.testing.assert_array_equal(g.rgb, want, err_msg=f"case {case} ({n} primitives, {per_obs} values, {src})")
            np.testing.assert_array_equal(g.depth.view(np.uint32), before.depth.view(np.uint32))
            if case % 2 == 0:
                assert (g.rgb[~obs_active] == 7).all()
            covered = np.zeros((H, W), bool)
            for x, y, w, h, *_ in rects:
                covered[y:y + h, x:x + w] = True
            np.testing.assert_array_equal(g.rgb[:, ~covered], before.rgb[:, ~covered])     # the render shows through
    # one rightward gauge is the bar
    run.batch.set_active(None)
    fractions = rng.uniform(-0.2, 1.2, size=spec.num_obs).astype(np.float32)
    run.render()
    run.batch.draw_bars(run.rgb, fractions, 8, 4, 100, 3, (255, 255, 0), (40, 40, 40), stream=_stream())
    torch.cuda.synchronize()
    with_bar = run.numpy().rgb.copy()
    run.render()
    run.batch.draw_overlay(run.rgb, [(8, 4, 100, 3, (255, 255, 0), binding.RECT_GAUGE_RIGHT, (40, 40, 40), 0)],
                           fractions.reshape(-1, 1), stream=_stream())
    torch.cuda.synchronize()
    np.testing.assert_array_equal(run.numpy().rgb, with_bar)
    # refusals
    ok = (0, 0, 4, 4, (1, 2, 3), 0, (0, 0, 0), 0)
    for rects, values in (([(W - 3, 0, 4, 4, (0, 0, 0), 0, (0, 0, 0), 0)], None),              # sticks out
                          ([(0, 0, 4, 4, (0, 0, 0), 3, (0, 0, 0), 0)], None),                  # unknown kind
                          ([(0, 0, 4, 4, (0, 0, 0), 1, (0, 0, 0), 0)], None),                  # a gauge without values
                          ([(0, 0, 4, 4, (0, 0, 0), 2, (0, 0, 0), 2)], np.zeros((spec.num_obs, 2), np.float32)),
                          ([ok] * 33, None),                                                   # too many primitives
                          ([ok], np.zeros((spec.num_obs, 9), np.float32)),                     # too many values
                          ([], None)):
        with pytest.raises(binding.MvError) as e:
            run.batch.draw_overlay(run.rgb, rects, values)
        assert e.value.code == binding.MV_ERR_ARG, (rects[:1], e.value.code)
    bad = np.zeros((spec.num_obs, 1), np.float32)
    bad[5, 0] = np.nan
    with pytest.raises(binding.MvError) as e:
        run.batch.draw_overlay(run.rgb, [(0, 0, 4, 4, (0, 0, 0), 1, (0, 0, 0), 0)], bad)
    assert e.value.code == binding.MV_ERR_ARG


def test_single_call_step_against_the_oracle(lib, orc):
    """mv_step = edits + cameras + finished-episode flags + render + bar + overlay in one call, device inputs only:
    three steps of the dynamic workload against the oracle; frames of finished environments keep what the
    tensors held; the flags of one step do not leak into the next."""
    wl = synth.generate(1, num_envs=12)
    spec = wl.spec
    rng = np.random.default_rng(5)
    X, Y, Z = spec.grid
    ob = _oracle_for(orc, spec, wl.voxels, wl.palette, wl.cameras[0])
    run = _gpu_for(spec, wl.voxels, wl.palette, wl.cameras[0], aux=False)
    bar = dict(x=4, y=2, width=64, height=2, fill_rgb=(0, 255, 0), empty_rgb=(10, 10, 10))
    # overlay: a frame part over the bar's right end, an upward gauge, and a mark on top of the gauge
    overlay = [(60, 1, 12, 5, (200, 200, 0), binding.RECT_SOLID, (0, 0, 0), 0),
               (100, 20, 6, 40, (255, 0, 0), binding.RECT_GAUGE_UP, (30, 30, 30), 1),
               (100, 38, 6, 2, (255, 255, 255), binding.RECT_SOLID, (0, 0, 0), 0)]
    vox = wl.voxels.copy()
    for step in range(3):
        # this step's edits: a few voxels per environment set or cleared (one edit per voxel)
        n = 40
        flat = rng.choice(spec.num_envs * X * Y * Z, size=n, replace=False)
        env, idx = (flat // (X * Y * Z)).astype(np.int32), (flat % (X * Y * Z)).astype(np.int32)
        mat = np.where(rng.random(n) < 0.5, 0, rng.integers(1, spec.num_materials + 1, size=n)).astype(np.uint8)
        cams = synth.random_cameras(rng, spec.num_obs, spec.grid, margin=0.0, max_pitch=0.6)
        selfv = None
        if step == 2:                        # every camera stands in a body of its own (its cell and the one above)
            cell = np.minimum(np.floor(cams[:, :3]).astype(np.int64), np.array([X - 1, Y - 1, Z - 1]))
            selfv = ((cell[:, 2] * Y + cell[:, 1]) * X + cell[:, 0]).astype(np.int32)
        done = (rng.random(spec.num_envs) < 0.3).astype(np.uint8) if step != 1 else None
        fractions = rng.uniform(0, 1, size=spec.num_obs).astype(np.float32)
        ob.update_voxels(env, idx, mat)
        ob.set_cameras(cams, selfv)
        ref = ob.render(threads=8)
        active = np.ones(spec.num_envs, np.uint8) if done is None else (done == 0).astype(np.uint8)
        want_rgb = ref.rgb.copy()
        ob.draw_bars(want_rgb, fractions, active=active, **bar)
        gauges = rng.uniform(-0.1, 1.1, size=(spec.num_obs, 2)).astype(np.float32)
        with_overlay = step != 0
        if with_overlay:
            ob.draw_overlay(want_rgb, overlay, gauges, active=active)
        run.rgb.fill_(7)
        run.depth.fill_(-1.0)
        dev = lambda a: None if a is None else torch.from_numpy(a).cuda()
        run.batch.step(dev(cams), run.rgb, run.depth, edits=(dev(env), dev(idx), dev(mat)), self_voxel=dev(selfv),
                       done=dev(done), bar_fraction=dev(fractions), bar=bar,
                       overlay=overlay if with_overlay else None, overlay_values=dev(gauges) if with_overlay else None,
                       stream=_stream())
        torch.cuda.synchronize()
        rgb, depth = run.rgb.cpu().numpy(), run.depth.cpu().numpy()
        obs_active = np.repeat(active.astype(bool), spec.agents_per_env)
        assert (rgb[~obs_active] == 7).all() and (depth[~obs_active] == -1.0).all()
        # depth and colours of the rendered frames: the parity rule without the side channels
        tie = ref.edge_margin < parity.EDGE_MARGIN
        ok = obs_active[:, None, None] & ~tie
        assert ((ref.depth == 0) == (depth == 0))[ok].all(), f"step {step}"
        assert (np.abs(depth - ref.depth)[ok] <= 1e-4 * np.abs(ref.depth)[ok]).all(), f"step {step}"
        assert (np.abs(rgb.astype(int) - want_rgb.astype(int)).max(axis=-1)[ok] <= 1).all(), f"step {step}"
        np.testing.assert_array_equal(rgb[obs_active][:, 2:4, 4:68], want_rgb[obs_active][:, 2:4, 4:68])
        if with_overlay:
            np.testing.assert_array_equal(rgb[obs_active][:, 1:6, 60:72], want_rgb[obs_active][:, 1:6, 60:72])
            np.testing.assert_array_equal(rgb[obs_active][:, 20:60, 100:106], want_rgb[obs_active][:, 20:60, 100:106])
        assert ok.mean() > 0.5
    # without edits, flags and bar the call is cameras + render
    run.batch.step(torch.from_numpy(wl.cameras[0]).cuda(), run.rgb, run.depth, stream=_stream())
    torch.cuda.synchronize()
    ob.set_cameras(wl.cameras[0], None)
    ref = ob.render(threads=8)
    ok = ~(ref.edge_margin < parity.EDGE_MARGIN)
    assert (np.abs(run.depth.cpu().numpy() - ref.depth)[ok] <= 1e-4 * np.abs(ref.depth)[ok]).all()
    with pytest.raises(binding.MvError) as e:
        run.batch.step(None, run.rgb, run.depth)
    assert e.value.code == binding.MV_ERR_ARG


def test_step_replays_from_a_hip_graph(lib, orc):
    """The device-source calls enqueue kernels only (no allocation, no synchronisation, no memset), so a
    step can be captured once into a HIP graph and replayed: every replay, with fresh cameras and
    voxel edits copied into the captured input buffers and eager work in between, must equal the
    eager result bit for bit."""
    wl = synth.generate(3, num_envs=64)
    spec = wl.spec
    batch = binding.Batch(spec.num_envs, spec.agents_per_env, spec.grid, spec.num_materials, spec.width, spec.height)
    eager = binding.Batch(spec.num_envs, spec.agents_per_env, spec.grid, spec.num_materials, spec.width, spec.height)
    vox, cams, selfv = wl.voxels, wl.cameras[0], wl.self_voxel[0]
    for b in (batch, eager):
        b.upload_worlds(vox, wl.palette)
    run_g, run_e = GpuRender(batch, spec.width, spec.height, aux=False), GpuRender(eager, spec.width, spec.height, aux=False)
    max_edits = 8192
    cams_in = torch.from_numpy(cams).cuda()
    self_in = torch.from_numpy(selfv).cuda()
    env_in = torch.full((max_edits,), -1, dtype=torch.int32, device="cuda")        # -1: dropped by the kernel
    idx_in = torch.zeros(max_edits, dtype=torch.int32, device="cuda")
    mat_in = torch.zeros(max_edits, dtype=torch.uint8, device="cuda")
    # an overlay in the captured step as well: the list is read at capture time, the gauge values at every replay
    overlay = [(2, 2, 40, 3, (0, 255, 0), binding.RECT_GAUGE_RIGHT, (20, 20, 20), 0),
               (120, 10, 4, 50, (255, 0, 0), binding.RECT_GAUGE_UP, (20, 20, 20), 1),
               (30, 1, 6, 5, (250, 250, 250), binding.RECT_SOLID, (0, 0, 0), 0)]
    gauges_in = torch.zeros((spec.num_obs, 2), dtype=torch.float32, device="cuda")
    gauge_rng = np.random.default_rng(77)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        batch.set_cameras(cams_in, self_in, stream=side.cuda_stream)                # warm-up outside the capture
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            st = torch.cuda.current_stream().cuda_stream
            # the single-call form of the step; the eager path below uses the separate calls
            batch.step(cams_in, run_g.rgb, run_g.depth, edits=(env_in, idx_in, mat_in), self_voxel=self_in,
                       overlay=overlay, overlay_values=gauges_in, stream=st)
    torch.cuda.synchronize()
    for step in range(1, 5):
        prev = vox
        vox, cams, selfv = synth.dynamic_step(wl)
        env, idx, mat = synth.grid_edits(prev, vox)
        assert env.size <= max_edits
        # eager reference path
        eager.update_voxels(torch.from_numpy(env).cuda(), torch.from_numpy(idx).cuda(), torch.from_numpy(mat).cuda(),
                            stream=_stream())
        eager.set_cameras(torch.from_numpy(cams).cuda(), torch.from_numpy(selfv).cuda(), stream=_stream())
        run_e.render()
        gauges = torch.from_numpy(gauge_rng.uniform(-0.1, 1.1, size=(spec.num_obs, 2)).astype(np.float32)).cuda()
        eager.draw_overlay(run_e.rgb, overlay, gauges, stream=_stream())
        # graph path: refresh the captured input buffers, replay
        env_in.fill_(-1)
        env_in[:env.size] = torch.from_numpy(env).cuda()
        idx_in[:env.size] = torch.from_numpy(idx).cuda()
        mat_in[:env.size] = torch.from_numpy(mat).cuda()
        cams_in.copy_(torch.from_numpy(cams).cuda())
        self_in.copy_(torch.from_numpy(selfv).cuda())
        gauges_in.copy_(gauges)
        run_g.rgb.fill_(7); run_g.depth.fill_(-1.0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(run_g.rgb, run_e.rgb), step
        assert torch.equal(run_g.depth.view(torch.int32), run_e.depth.view(torch.int32)), step
    ob = _oracle_for(orc, spec, vox, wl.palette, cams, selfv)
    ref = ob.render(threads=8)
    g = run_g.numpy()
    covered = np.zeros((spec.height, spec.width), bool)
    for x, y, w, h, *_ in overlay:
        covered[y:y + h, x:x + w] = True
    want = ref.rgb.copy()
    ob.draw_overlay(want, overlay, gauges.cpu().numpy())
    np.testing.assert_array_equal(g.rgb[:, covered], want[:, covered])      # the primitives, byte for byte
    g.rgb[:, covered] = ref.rgb[:, covered]                                 # and every other pixel under the parity rule
    parity.compare(g, ref, label="graph replay, last step")


# ------------------------------------------------------------------------------------------ the other render paths, at scale
@pytest.mark.parametrize("name", ["wide", "outside", "odd"])
def test_slow_paths_on_mid_size_batches(lib, orc, name):
    """Every pixel against the oracle on batches of hundreds of observations for the paths the five workloads
    never take: grids wider than 64 voxels (per-cell tracer over rows on chip), cameras outside the grid (per-cell
    tracer over rows in device memory), and an image that is not made of whole 8x8 tiles (clamped tiles, byte
    stores) -- several workgroups per compute unit, tail strips and the XCD mapping included."""
    wl = synth.generate_extra(name)
    spec = wl.spec
    ob = _oracle_for(orc, spec, wl.voxels, wl.palette, wl.cameras[0])
    run = _gpu_for(spec, wl.voxels, wl.palette, wl.cameras[0])
    run.render()
    st = _compare_all(ob, run, label=name, chunk=256)
    assert st["pixels"] == spec.num_obs * spec.height * spec.width
    if name == "outside":
        assert (run.depth > 0).float().mean().item() > 0.2          # the cameras do look at their arenas


def test_step_captured_over_low_worlds_replays_over_taller_ones(lib, orc):
    """A graph captured while every world is two layers tall must still render at full speed, and correctly,
    when taller worlds are uploaded afterwards: the captured launch reserves room for all layers instead of the
    number that happened to be enough at capture time.  Replay vs oracle, and replay time vs the eager call, on
    the benchmark's batch (4096 environments x 2 agents: a step long enough that the few microseconds a replay
    costs by itself do not decide the comparison)."""
    wl = synth.generate(2, steps=1)
    spec = wl.spec
    low = wl.voxels.copy()
    low[:, 2:] = 0                                                  # floor + one layer of walls
    batch = binding.Batch(spec.num_envs, spec.agents_per_env, spec.grid, spec.num_materials, spec.width, spec.height)
    run = GpuRender(batch, spec.width, spec.height, aux=False)
    low_d, tall_d = torch.from_numpy(low).cuda(), torch.from_numpy(wl.voxels).cuda()
    pal_d = torch.from_numpy(wl.palette).cuda()
    cams_in = torch.from_numpy(wl.cameras[0]).cuda()
    batch.upload_worlds(low_d, pal_d, stream=_stream())
    batch.set_cameras(cams_in, stream=_stream())
    run.render()
    torch.cuda.synchronize()                                        # the host has now heard: worlds are 2 layers tall
    run.render()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            batch.step(cams_in, run.rgb, run.depth, stream=torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    graph.replay()
    torch.cuda.synchronize()
    ob_low = _oracle_for(orc, spec, low, wl.palette, wl.cameras[0])
    _compare_all(ob_low, run, label="replay over the low worlds", chunk=512)
    # taller worlds arrive
    batch.upload_worlds(tall_d, pal_d, stream=_stream())
    torch.cuda.synchronize()
    run.rgb.fill_(7); run.depth.fill_(-1.0)
    graph.replay()
    torch.cuda.synchronize()
    ob = _oracle_for(orc, spec, wl.voxels, wl.palette, wl.cameras[0])
    _compare_all(ob, run, label="replay over the taller worlds", chunk=512)

    def timed(fn, reps=100):
        for _ in range(30):
            fn()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        a.record()
        for _ in range(reps):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / reps
    t_eager = timed(lambda: batch.step(cams_in, run.rgb, run.depth, stream=_stream()))
    t_graph = timed(graph.replay)
    # Room for all layers costs a workgroup or two per compute unit against the eager call's ten layers; the path
    # through device memory that a frozen two-layer choice would take is several times slower.
    assert t_graph <= 1.10 * t_eager, (t_graph, t_eager)
    # a caller who knows how tall the worlds can get fixes the number before capturing: then the replay runs the
    # very launch the eager call makes
    batch.debug_set_staged_layers(10)
    pinned = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(pinned, stream=side):
            batch.step(cams_in, run.rgb, run.depth, stream=torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    run.rgb.fill_(7); run.depth.fill_(-1.0)
    pinned.replay()
    torch.cuda.synchronize()
    _compare_all(ob, run, label="replay with a fixed layer count", chunk=512)
    t_pinned = timed(pinned.replay)
    assert t_pinned <= 1.05 * t_eager, (t_pinned, t_eager)
    batch.debug_set_staged_layers(0)


def test_objects_moved_from_their_positions(lib, orc):
    """mv_move_voxels: the dynamic workload's boxes and agent bodies re-stamped from (old cell, new cell, material)
    lists -- no grid diff on the host.  After every step the batch must render what a batch with the freshly
    uploaded grid renders, bit for bit, and what the oracle renders from that grid; device and host lists alike.
    Objects follow each other and swap into vacated cells within one call."""
    wl = synth.generate(3, num_envs=96)
    spec = wl.spec
    moved = _gpu_for(spec, wl.voxels, wl.palette, wl.cameras[0], wl.self_voxel[0])
    fresh = _gpu_for(spec, wl.voxels, wl.palette, wl.cameras[0], wl.self_voxel[0])
    followed = 0
    for step in range(5):
        before = synth.dynamic_positions(wl)
        vox, cams, selfv = synth.dynamic_step(wl)
        after = synth.dynamic_positions(wl)
        env, frm, to, mat = synth.object_moves(wl, before, after)
        # cells that one object left and another entered in this very step
        left = set(zip(env[frm != to].tolist(), frm[frm != to].tolist()))
        followed += len(left & set(zip(env[frm != to].tolist(), to[frm != to].tolist())))
        if step % 2 == 0:
            moved.batch.move_voxels(*(torch.from_numpy(a).cuda() for a in (env, frm, to, mat)), stream=_stream())
        else:
            moved.batch.move_voxels(env, frm, to, mat, stream=_stream())
        cams_d, self_d = torch.from_numpy(cams).cuda(), torch.from_numpy(selfv).cuda()
        moved.batch.set_cameras(cams_d, self_d, stream=_stream())
        fresh.batch.upload_worlds(torch.from_numpy(vox).cuda(), None, stream=_stream())
        fresh.batch.set_cameras(cams_d, self_d, stream=_stream())
        moved.render()
        fresh.render()
        a, b = moved.numpy(), fresh.numpy()
        for name in ("rgb", "depth", "material", "hit_index", "face"):
            np.testing.assert_array_equal(getattr(a, name).view(np.uint8), getattr(b, name).view(np.uint8),
                                          err_msg=f"step {step} {name}")
        ob = _oracle_for(orc, spec, vox, wl.palette, cams, selfv)
        _compare_all(ob, moved, label=f"moved objects, step {step}", chunk=192)
    assert followed > 0                      # the case the clears-before-fills order exists for did occur
    with pytest.raises(binding.MvError) as err:
        moved.batch.move_voxels(np.array([0], np.int32), np.array([spec.grid[0] * spec.grid[1] * spec.grid[2]], np.int32),
                                np.array([0], np.int32), np.array([1], np.uint8))
    assert err.value.code == binding.MV_ERR_RANGE


def test_an_object_enters_the_voxel_another_one_leaves_in_the_same_call(lib, orc):
    """One edit list that empties a voxel and fills the same voxel again (object 1 leaves, object 2 enters),
    next to ordinary moves: clears are applied before fills whatever their order in the list, so the voxel ends
    up solid with the new material, its occupancy bit set -- as the oracle's in-order edits give for the order
    (clear, fill), and the same for the order (fill, clear) of a per-object list."""
    wl = synth.generate(1, num_envs=8)
    spec = wl.spec
    X, Y, Z = spec.grid
    vox = wl.voxels.copy()
    cams = wl.cameras[0]
    # put a box right in front of camera 0 of every environment, then swap it for a box of another material
    env, idx, mat_old, mat_new = [], [], [], []
    for n in range(spec.num_envs):
        c = cams[n * spec.agents_per_env]
        i, j = int(c[0]), int(c[1])
        for di, dj in ((1, 0), (-1, 0), (0, 1), (0, -1)):
            ii, jj = i + 2 * di, j + 2 * dj
            if 1 <= ii < X - 1 and 1 <= jj < Y - 1 and vox[n, 1, jj, ii] == 0:
                env.append(n); idx.append((1 * Y + jj) * X + ii); mat_old.append(3); mat_new.append(9)
                vox[n, 1, jj, ii] = 3
                break
    assert len(env) >= 4
    env = np.array(env, np.int32); idx = np.array(idx, np.int32)
    run = _gpu_for(spec, vox, wl.palette, cams)
    ob = _oracle_for(orc, spec, vox, wl.palette, cams)
    for order in ("clear first", "fill first"):
        clear = (env, idx, np.zeros(len(env), np.uint8))
        fill = (env, idx, np.array(mat_new, np.uint8))
        first, second = (clear, fill) if order == "clear first" else (fill, clear)
        e = np.concatenate([first[0], second[0]]); v = np.concatenate([first[1], second[1]])
        m = np.concatenate([first[2], second[2]])
        run.batch.update_voxels(torch.from_numpy(e).cuda(), torch.from_numpy(v).cuda(), torch.from_numpy(m).cuda(),
                                stream=_stream())
        ob.update_voxels(*clear)                                    # the oracle applies edits in list order
        ob.update_voxels(*fill)
        run.render()
        st = parity.compare(run.numpy(), ob.render(threads=8), label=order)
        assert st["pixels"] > 0
        hit_new = run.numpy().material == 9
        assert hit_new.any(), order                                 # the new boxes are seen, with their material
        # back to the old material for the second order
        back = (env, idx, np.array(mat_old, np.uint8))
        run.batch.update_voxels(*(torch.from_numpy(a).cuda() for a in back), stream=_stream())
        ob.update_voxels(*back)


def test_upload_of_the_largest_layer_the_pack_kernel_holds(lib, orc):
    """200x200x2: each of the pack kernel's four waves keeps a whole 40,000-byte layer in LDS, just under the
    limit checked at creation; the packed rows and a small render must be right."""
    grid = (200, 200, 2)
    rng = np.random.default_rng(11)
    N, A, M = 2, 2, 5
    spec = _mini_spec(N, A, grid, 64, 40, M)
    vox, pal = synth.random_world(rng, N, grid, 0.05, M)
    vox[:, 0] = np.where(vox[:, 0] == 0, 1, vox[:, 0])               # a floor
    cams = synth.random_cameras(rng, N * A, grid, margin=0.0, max_pitch=0.6)
    cams[:, 2] = 1.5
    for o in range(N * A):
        vox[o // A, 1, int(cams[o, 1]), int(cams[o, 0])] = 0           # the cameras stand in empty cells
    ob = _oracle_for(orc, spec, vox, pal, cams)
    run = _gpu_for(spec, vox, pal, cams)
    run.render()
    parity.compare(run.numpy(), ob.render(threads=8), label="200x200x2")


def test_coarse_level_gives_the_same_bits(lib, orc):
    """coarse_level = 1 (long rays look at the OR of pairs of rows first) must not change a single output bit:
    colour, depth, material, hit index and face against the default kernel, on structured batches with own
    bodies, on grids with odd row counts, and against the oracle."""
    cases = []
    wl = synth.generate(1)
    cases.append((wl.spec, wl.voxels, wl.palette, wl.cameras[0], None))
    dyn = synth.generate(3, num_envs=48)
    cases.append((dyn.spec, dyn.voxels, dyn.palette, dyn.cameras[0], dyn.self_voxel[0]))
    rng = np.random.default_rng(21)
    for grid in ((39, 41, 7), (64, 63, 5), (5, 3, 9), (33, 2, 4)):
        N, A, M = 6, 3, 5
        spec = _mini_spec(N, A, grid, 72, 40, M)
        vox, pal = synth.random_world(rng, N, grid, 0.04, M)
        cams = synth.random_cameras(rng, N * A, grid, margin=0.0, max_pitch=1.2)
        cases.append((spec, vox, pal, cams, None))
    for spec, vox, pal, cams, selfv in cases:
        plain = _gpu_for(spec, vox, pal, cams, selfv)
        coarse = _gpu_for(spec, vox, pal, cams, selfv, coarse_level=1)
        plain.render()
        coarse.render()
        a, b = plain.numpy(), coarse.numpy()
        for name in ("rgb", "depth", "material", "hit_index", "face"):
            np.testing.assert_array_equal(getattr(a, name).view(np.uint8), getattr(b, name).view(np.uint8),
                                          err_msg=f"{spec.grid} {name}")
        ob = _oracle_for(orc, spec, vox, pal, cams, selfv)
        _compare_all(ob, coarse, label=f"coarse level {spec.grid}", chunk=256)


# ------------------------------------------------------------------------------------------ pieces
def _read_device(ptr, nbytes):
    hip = C.CDLL("libamdhip64.so")
    hip.hipMemcpy.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_int]
    buf = np.empty(nbytes, np.uint8)
    assert hip.hipMemcpy(buf.ctypes.data, ptr, nbytes, 2) == 0
    return buf


@pytest.mark.parametrize("grid", [(40, 40, 16), (7, 5, 3), (16, 16, 8), (64, 64, 4), (70, 3, 5), (3, 130, 2), (64, 64, 9),
                                  (48, 56, 10), (36, 20, 7)])
def test_pack_kernel_bit_exact(lib, grid):
    """Occupancy bit rows along x and along y, and the top solid layer, against NumPy: after a first upload,
    after a single voxel set high up, and after re-uploads of lower and of taller worlds (empty layers at
    and above the previous top are skipped by the kernel and must still read as zero)."""
    rng = np.random.default_rng(17)
    N = 6
    X, Y, Z = grid
    batch = binding.Batch(N, 1, grid, 4, 16, 8)

    def check(vox, top_is_exact=True):
        torch.cuda.synchronize()
        for env in range(N):
            xp, xw, yp, yw, tp = batch.debug_occupancy(env)
            assert xw == (X + 63) // 64 and yw == (Y + 63) // 64
            occ = vox[env] != 0                                               # [Z,Y,X]
            want_x = np.packbits(np.pad(occ, ((0, 0), (0, 0), (0, xw * 64 - X))), axis=-1, bitorder="little")
            got_x = _read_device(xp, Z * Y * xw * 8).reshape(Z, Y, xw * 8)
            np.testing.assert_array_equal(got_x, want_x)
            occ_t = occ.transpose(0, 2, 1)                                    # [Z,X,Y]
            want_y = np.packbits(np.pad(occ_t, ((0, 0), (0, 0), (0, yw * 64 - Y))), axis=-1, bitorder="little")
            got_y = _read_device(yp, Z * X * yw * 8).reshape(Z, X, yw * 8)
            np.testing.assert_array_equal(got_y, want_y)
            layers = np.nonzero(occ.any(axis=(1, 2)))[0]
            top = int(_read_device(tp, 4).view(np.int32)[0])
            exact = int(layers.max()) + 1 if layers.size else 0
            assert top == exact if top_is_exact else top >= exact

    vox, pal = synth.random_world(rng, N, grid, 0.3, 4)
    vox[3, Z // 2:] = 0                       # environment 3: empty upper half
    vox[N - 1] = 0                            # last environment: empty
    batch.upload_worlds(torch.from_numpy(vox).cuda(), torch.from_numpy(pal).cuda(), stream=_stream())
    check(vox)
    # one voxel set in the top layer of the half-empty and of the empty environment
    idx = ((Z - 1) * Y + (Y - 1)) * X + (X - 1)
    batch.update_voxels(np.array([3, N - 1], np.int32), np.array([idx, idx], np.int32), np.array([2, 1], np.uint8))
    vox[3].reshape(-1)[idx] = 2
    vox[N - 1].reshape(-1)[idx] = 1
    check(vox)
    # lower worlds everywhere (the rows of the layers that were solid must be cleared), then taller ones again
    for keep in (max(Z // 3, 1), Z, 0, max(Z // 2, 1)):
        vox2, _ = synth.random_world(rng, N, grid, 0.3, 4)
        vox2[:, keep:] = 0
        vox2[1] = 0
        batch.upload_worlds(torch.from_numpy(vox2).cuda(), None, stream=_stream())
        check(vox2)
        vox3, _ = synth.random_world(rng, 2, grid, 0.2, 4)      # partial upload from host memory
        batch.upload_worlds(vox3, None, first_env=2)
        vox2[2:4] = vox3
        check(vox2)


def test_camera_records_match_the_oracle(lib, orc):
    rng = np.random.default_rng(23)
    N, A = 64, 4
    grid = (40, 40, 16)
    cams = synth.random_cameras(rng, N * A, grid)
    selfv = rng.integers(-1, 40 * 40 * 15, size=N * A).astype(np.int32)
    batch = binding.Batch(N, A, grid, 3)
    batch.set_cameras(torch.from_numpy(cams).cuda(), torch.from_numpy(selfv).cuda(), stream=_stream())
    torch.cuda.synchronize()
    raw = _read_device(batch.debug_camera_records(), N * A * 64)
    rec_f = raw.view(np.float32).reshape(N * A, 16)
    rec_i = raw.view(np.int32).reshape(N * A, 16)
    ob = orc.OracleBatch(N, A, grid, 128, 72, 3)
    ob.set_cameras(cams, selfv)
    want = np.stack([ob.camera_record(o) for o in range(N * A)])
    ulp = np.abs(rec_f[:, :12].view(np.int32).astype(np.int64) - want.view(np.int32).astype(np.int64))
    # float64 sin/cos of two math libraries may differ in the last bit before rounding to float32
    assert ulp.max() <= 1 and (ulp == 0).mean() > 0.999
    np.testing.assert_array_equal(rec_i[:, 12], selfv)
    np.testing.assert_array_equal(rec_i[:, 13], np.where(selfv >= 0, selfv + 1600, -1))
