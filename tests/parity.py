"""Comparison rule between the HIP library's output and the CPU oracle, and a certificate that
checks any renderer output against the scene without a second renderer.

Rule (from the project's stated tolerances): material id, hit-voxel index and entered face are
bit-exact on at least 99.95 % of pixels; a differing pixel is admissible only if the oracle's ray
passed within 1e-4 voxel of a voxel edge (float32 cannot resolve finer); on agreeing pixels colour
is within 1 LSB per channel, depth within 1e-4 relative, and misses are bit-exact.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

EDGE_MARGIN = 1e-4
MIN_EXACT_FRACTION = 0.9995
DEPTH_RTOL = 1e-4


@dataclass
class GpuOut:
    rgb: np.ndarray
    depth: np.ndarray
    material: np.ndarray = None
    hit_index: np.ndarray = None
    face: np.ndarray = None


def compare(gpu: GpuOut, ref, sky_rgb=(135, 206, 235), label: str = "") -> dict:
    """Assert the rule; returns statistics.  ``ref`` is an oracle ``Rendered`` over the same pixels."""
    assert gpu.rgb.shape == ref.rgb.shape and gpu.depth.shape == ref.depth.shape, label
    n = ref.depth.size
    if gpu.hit_index is not None:
        differ = (gpu.hit_index != ref.hit_index) | (gpu.material != ref.material) | (gpu.face != ref.face)
    else:
        # colour/depth-only outputs: a pixel "differs" when colour is off by more than 1 LSB or depth by
        # more than the tolerance; the same admissibility rule applies
        drgb = np.abs(gpu.rgb.astype(np.int16) - ref.rgb.astype(np.int16)).max(axis=-1)
        differ = (drgb > 1) | (np.abs(gpu.depth - ref.depth) > DEPTH_RTOL * np.abs(ref.depth))
    frac_exact = 1.0 - differ.mean()
    bad = differ & ~(ref.edge_margin < EDGE_MARGIN)
    assert not bad.any(), (f"{label}: {int(bad.sum())} pixels differ away from any voxel edge, first at "
                           f"{tuple(np.argwhere(bad)[0])}")
    assert frac_exact >= MIN_EXACT_FRACTION, f"{label}: only {frac_exact:.6f} of pixels exact"
    same = ~differ
    drgb = np.abs(gpu.rgb.astype(np.int16) - ref.rgb.astype(np.int16)).max(axis=-1)
    assert (drgb[same] <= 1).all(), f"{label}: colour off by {int(drgb[same].max())} LSB"
    hit = same & (ref.hit_index >= 0)
    rel = np.abs(gpu.depth[hit].astype(np.float64) - ref.depth[hit]) / np.maximum(ref.depth[hit], 1e-30)
    # depth 0 (origin inside a solid) must be exactly 0
    zero = ref.depth[hit] == 0
    assert (gpu.depth[hit][zero] == 0).all(), label
    max_rel = float(rel[~zero].max()) if (~zero).any() else 0.0
    assert max_rel <= DEPTH_RTOL, f"{label}: depth relative error {max_rel:.3e}"
    miss = same & (ref.hit_index < 0)
    assert (gpu.depth[miss].view(np.uint32) == 0).all(), f"{label}: miss depth not +0.0"
    assert (gpu.rgb[miss] == np.array(sky_rgb, np.uint8)).all(), f"{label}: miss colour is not the sky"
    return {"pixels": int(n), "exact_fraction": float(frac_exact), "differ": int(differ.sum()),
            "max_depth_rel": max_rel, "max_rgb_lsb": int(drgb[same].max()) if same.any() else 0,
            "colour_exact_fraction": float((drgb[same] == 0).mean()) if same.any() else 1.0}


def certificate(orc, oracle_batch, vox_env: np.ndarray, obs: int, gpu: GpuOut, local: int, rng, samples: int = 300,
                self_voxel: int = -1) -> int:
    """Check GPU pixels of one observation against the scene itself: the claimed hit point
    P + depth*d lies on the claimed face of the claimed voxel, that voxel is solid, and the
    brute-force definition finds no solid voxel nearer.  Returns the number of pixels checked."""
    X, Y, Z = oracle_batch.grid
    H, W = oracle_batch.H, oracle_batch.W
    rec = oracle_batch.camera_record(obs).astype(np.float64)
    P = rec[:3]
    rows = rng.integers(0, H, size=samples)
    cols = rng.integers(0, W, size=samples)
    rays = np.empty((samples, 3), np.float64)
    full = None
    for s in range(samples):
        if full is None:
            full = oracle_batch.pixel_rays(obs).astype(np.float64)
        rays[s] = full[rows[s], cols[s]]
    hit, face, t = orc.definition_first_hit((X, Y, Z), vox_env, np.broadcast_to(P, rays.shape), rays,
                                            np.full(samples, self_voxel, np.int32))
    checked = 0
    for s in range(samples):
        r, c = rows[s], cols[s]
        g_idx = int(gpu.hit_index[local, r, c])
        g_face = int(gpu.face[local, r, c])
        g_t = float(gpu.depth[local, r, c])
        if g_idx < 0:
            if hit[s] >= 0:
                # admissible only when the definition's hit is a graze: the ray touches the voxel for a
                # tiny stretch (edge tie)
                pt = P + t[s] * rays[s]
                frac = np.abs(pt - np.round(pt))
                assert np.sort(frac)[1] < EDGE_MARGIN * 10, (obs, r, c, "GPU missed a voxel the ray clearly meets")
            continue
        k, rem = divmod(g_idx, X * Y)
        j, i = divmod(rem, X)
        assert vox_env[k, j, i] != 0, (obs, r, c, "claimed voxel is empty")
        assert int(gpu.material[local, r, c]) == int(vox_env[k, j, i])
        pt = P + g_t * rays[s]
        lo = np.array([i, j, k], np.float64)
        if g_face == 6:
            assert g_t == 0.0 and (P >= lo - 1e-6).all() and (P <= lo + 1 + 1e-6).all()
        else:
            axis, positive = divmod(g_face, 2)
            plane = lo[axis] + (1.0 if positive else 0.0)
            tol = 1e-4 * max(1.0, g_t)
            assert abs(pt[axis] - plane) <= tol, (obs, r, c, "hit point is not on the claimed face")
            for a in range(3):
                if a != axis:
                    assert lo[a] - tol <= pt[a] <= lo[a] + 1 + tol, (obs, r, c, "hit point outside the face")
            # the ray must be entering: direction against the outward normal
            assert (rays[s][axis] < 0) == bool(positive)
        # nothing nearer (brute force); ties within float32 resolution are admissible
        if hit[s] >= 0 and hit[s] != g_idx:
            assert t[s] >= g_t - 1e-4 * max(1.0, g_t), (obs, r, c, "a nearer solid voxel exists")
        assert hit[s] >= 0, (obs, r, c, "definition finds no voxel on this ray")
        checked += 1
    return checked
