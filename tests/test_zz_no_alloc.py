"""mv_render_worlds_noalloc (the entry point for callers that cannot allocate device memory) against the batch
path it is a variant of: mv_create_batch + mv_upload_worlds + mv_set_cameras + mv_render_batch.  Same kernels, same
inputs: colour and depth must agree bit for bit; the small second call is compared with the CPU oracle as well.
Calls in a row with the second smaller than the first, so that whatever the first call left in the library's
fixed scratch array would show."""
import ctypes as C

import numpy as np
import pytest

from paper_2107_08170_amd import binding, synth
from tests import parity

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def _stream():
    return torch.cuda.current_stream().cuda_stream


def _both_ways(num_envs, agents, grid, num_materials, W, H, voxels, palette, cams, self_voxel):
    """(rgb, depth) of the no-alloc call and of the batch path on the same device inputs."""
    dev = torch.device("cuda", 0)
    vox_d = torch.from_numpy(np.ascontiguousarray(voxels)).to(dev)
    pal_d = torch.from_numpy(np.ascontiguousarray(palette)).to(dev)
    cams_d = torch.from_numpy(np.ascontiguousarray(cams)).to(dev)
    self_d = None if self_voxel is None else torch.from_numpy(np.ascontiguousarray(self_voxel)).to(dev)
    n = num_envs * agents
    cfg = binding.make_config(num_envs, agents, grid, num_materials, W, H)
    rgb = torch.full((n, H, W, 3), 7, dtype=torch.uint8, device=dev)          # poisoned outputs
    depth = torch.full((n, H, W), -1.0, dtype=torch.float32, device=dev)
    binding.render_worlds_noalloc(cfg, vox_d, pal_d, cams_d, self_d, rgb, depth, stream=_stream())
    torch.cuda.synchronize()
    batch = binding.Batch(num_envs, agents, grid, num_materials, W, H)
    rgb2 = torch.full((n, H, W, 3), 9, dtype=torch.uint8, device=dev)
    depth2 = torch.full((n, H, W), -2.0, dtype=torch.float32, device=dev)
    batch.upload_worlds(vox_d, pal_d, stream=_stream())
    batch.set_cameras(cams_d, self_d, stream=_stream())
    batch.render(rgb2, depth2, stream=_stream())
    torch.cuda.synchronize()
    batch.close()
    return (rgb.cpu().numpy(), depth.cpu().numpy()), (rgb2.cpu().numpy(), depth2.cpu().numpy())


def _same_bits(a, b, label):
    np.testing.assert_array_equal(a[0], b[0], err_msg=f"{label}: colour")
    np.testing.assert_array_equal(a[1].view(np.uint32), b[1].view(np.uint32), err_msg=f"{label}: depth")
    assert (a[1] >= 0).all(), f"{label}: a pixel was never written"


def test_noalloc_entry_point_equals_the_batch_path_on_calls_in_a_row():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU")
    binding.load_library()
    # first call: 256 environments x 4 agents of 40x40x16 voxels (2.8 MB of the 8 MiB scratch array)
    big = synth.generate(1)
    s = big.spec
    a, b = _both_ways(s.num_envs, s.agents_per_env, s.grid, s.num_materials, s.width, s.height, big.voxels, big.palette,
                      big.cameras[0], None)
    _same_bits(a, b, "256x4")
    assert (a[1] > 0).mean() > 0.5
    # second call, smaller: 4 environments x 1 agent of 16x16x8 voxels
    small = synth.generate(0)
    s = small.spec
    c, d = _both_ways(s.num_envs, s.agents_per_env, s.grid, s.num_materials, s.width, s.height, small.voxels,
                      small.palette, small.cameras[0], None)
    _same_bits(c, d, "4x1")
    # ... and against the oracle, under the rule every GPU result is held to
    from oracle import oracle as orc
    ob = orc.OracleBatch(s.num_envs, s.agents_per_env, s.grid, s.width, s.height, s.num_materials)
    ob.upload_worlds(small.voxels, small.palette)
    ob.set_cameras(small.cameras[0])
    stats = parity.compare(parity.GpuOut(c[0], c[1]), ob.render(), label="noalloc 4x1")
    assert stats["exact_fraction"] >= parity.MIN_EXACT_FRACTION
    # third call, in between in size: own bodies through self_voxel (96 environments of the dynamic workload), odd image
    dyn = synth.generate(3)
    s = dyn.spec
    envs = 96
    e, f = _both_ways(envs, s.agents_per_env, s.grid, s.num_materials, 100, 60, dyn.voxels[:envs], dyn.palette[:envs],
                      dyn.cameras[0][: envs * s.agents_per_env], dyn.self_voxel[0][: envs * s.agents_per_env])
    _same_bits(e, f, "96x4 with own bodies")


def test_noalloc_entry_point_refuses_what_does_not_fit():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU")
    lib = binding.load_library()
    cfg = binding.make_config(4096, 2, (40, 40, 16), 16)                 # 42 MB of bit rows: beyond the scratch array
    rc = lib.mv_render_worlds_noalloc(C.byref(cfg), 1, 1, 1, None, 4, 4, None)
    assert rc == binding.MV_ERR_CAPACITY and b"scratch" in lib.mv_last_error()
