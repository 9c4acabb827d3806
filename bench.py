#!/usr/bin/env python3
"""Benchmark of the batched egocentric render on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 2]

A step is one pass of the whole hot path over one batch of synthetic input that is already
resident in device memory: world upload + occupancy packing + colour tables (mv_upload_worlds),
camera records (mv_set_cameras, a fresh camera set every step) and the render
(mv_render_batch) of every observation.  Prints ONE JSON line: observations/s (whole job), the
roofline of the dominant kernel measured with HIP events around every render launch, and the CPU
oracle timed on a bounded sample of the same workload on the host cores.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E datasheet peak
# Vector-ALU peak: the published 157.3 TFLOP/s fp32 vector figure with a fused multiply-add counted as ONE
# lane-instruction: 256 CUs x 4 SIMDs x 32 lanes x 2.4 GHz.  Only the full-rate instructions (fma, add,
# multiply, move, and, right shifts) can reach it; min/max, compares, selects, conversions and 64-bit shifts
# issue at half of it (profiles/valu_instruction_rates.txt), and they are most of a ray traversal.
ALU_PEAK_GOPS = 256 * 4 * 32 * 2.4     # 78643.2 G lane-instructions/s
# Mean per-cell DDA steps per ray of the CPU oracle on camera set 0 of each workload (measured with the
# oracle's step counter on the first 256/512/256/128 environments); the cpu_baseline leg re-measures it.
ORACLE_MEAN_STEPS = {1: 8.75, 2: 8.98, 3: 8.45, 4: 10.20}


def algorithmic_lane_ops_per_ray(mean_steps: float) -> float:
    """ALU work a plain per-cell DDA ray caster cannot do without, per ray: 10 lane-instructions per step
    (select the nearest plane, advance the cell, recompute that crossing, address and test one bit) plus
    60 fixed (ray set-up with three reciprocals, hit point and face, shading look-up, stores): the low
    ends of the ranges a hand count gives (10-15 and 60-100)."""
    return 10.0 * mean_steps + 60.0


def algorithmic_bytes_per_obs(spec) -> float:
    """HBM bytes the render of one observation must move: 7 bytes written per ray (3 colour +
    4 depth), 1 material byte read per ray at the hit, the environment's occupancy bits and colour
    table once per environment (shared by its A agents), one 64-byte camera record."""
    X, Y, Z = spec.grid
    rays = spec.width * spec.height
    occ_bytes = ((X * Y * Z + 31) // 32) * 4
    lut_bytes = 7 * (spec.num_materials + 1) * 4
    return rays * 7 + rays * 1 + (occ_bytes + lut_bytes) / spec.agents_per_env + 64


def measured_traffic(workload: str, column: int = 1):
    """Bytes per render launch from the committed rocprofv3 counter summary: column 1 = HBM (FETCH_SIZE and
    WRITE_SIZE scaled against a plain copy), column 2 = LDS (from SQ_INSTS_LDS); None when no summary covers
    this workload.  Column 3 = vector lane-instructions executed per launch (SQ_INSTS_VALU x 64)."""
    path = os.path.join(ROOT, "profiles", "render_traffic.txt")
    try:
        with open(path) as f:
            for line in f:
                parts = line.split()
                if len(parts) > column and parts[0] == workload:
                    return float(parts[column])
    except OSError:
        pass
    return None


def input_digest(wl) -> str:
    """SHA-256 over the generated grids, palettes and cameras: identifies the synthetic input of a run."""
    import hashlib
    import numpy as np
    h = hashlib.sha256()
    for a in (wl.voxels, wl.palette, wl.cameras):
        h.update(np.ascontiguousarray(a).data)
    return h.hexdigest()


def device_copy_rate(torch) -> float:
    """Read + written GB/s of a plain 512 MiB device-to-device copy: what HBM delivers to a streaming
    kernel on this GPU, quoted next to the 8 TB/s datasheet peak."""
    nbytes = 512 << 20
    src = torch.full((nbytes,), 5, dtype=torch.uint8, device="cuda")
    dst = torch.empty_like(src)
    dst.copy_(src)
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(5):
        dst.copy_(src)
    b.record()
    torch.cuda.synchronize()
    return 2.0 * nbytes * 5 / (a.elapsed_time(b) * 1e-3) / 1e9


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    # defaults: the shader clock needs about a hundred launches after idle to settle (the first launches of a
    # run are up to 25 % slower), so the warm-up covers that and the timed region is long enough to average
    # the rest out; the whole timed region still lasts well under a second
    ap.add_argument("--steps", type=int, default=500)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--config", type=int, default=2, help="workload index 1..4 (default 2: 4096 envs x 2 agents)")
    ap.add_argument("--tiles-per-block", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-envs", type=int, default=4096)
    ap.add_argument("--static-worlds", action="store_true",
                    help="upload the worlds once instead of every step (not the headline number)")
    ap.add_argument("--sparse-edits", action="store_true",
                    help="dynamic workload only: send the changed voxels of each step with mv_update_voxels instead "
                         "of re-uploading whole grids")
    ap.add_argument("--traffic-calibration", action="store_true",
                    help="run only a plain 1 GiB device-to-device copy five times, for scaling the HBM byte "
                         "counters of a rocprofv3 --pmc run against a kernel of known traffic")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (environments are independent; "
              "a second GPU would simply own other environments). Run with --gpus 1.", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    import paper_2107_08170_amd as mv
    from paper_2107_08170_amd import synth

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        return 2
    if args.traffic_calibration:
        nbytes = 1 << 30
        src = torch.full((nbytes,), 3, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibration": "device copy", "bytes_read": nbytes, "bytes_written": nbytes, "repeats": 5}))
        return 0
    mv.load_library()

    spec = synth.SPECS[args.config]
    t0 = time.time()
    wl = synth.generate(args.config)
    gen_s = time.time() - t0
    dev = torch.device("cuda", 0)
    stream = torch.cuda.current_stream().cuda_stream
    batch = mv.Batch(spec.num_envs, spec.agents_per_env, spec.grid, spec.num_materials, spec.width, spec.height,
                     tiles_per_block=args.tiles_per_block)
    vox_d = torch.from_numpy(wl.voxels).to(dev)
    pal_d = torch.from_numpy(wl.palette).to(dev)
    n_sets = max(1, spec.steps)
    if spec.dynamic:
        # dynamic worlds: pre-compute the grids/cameras of a few steps on the host, keep them resident
        n_sets = 4
        grids, cams_l, self_l = [wl.voxels], [wl.cameras[0]], [wl.self_voxel[0]]
        for _ in range(n_sets - 1):
            g, c, s = synth.dynamic_step(wl)
            grids.append(g); cams_l.append(c); self_l.append(s)
        grids_d = [torch.from_numpy(g).to(dev) for g in grids]
        cams_d = torch.from_numpy(np.stack(cams_l)).to(dev)
        self_d = torch.from_numpy(np.stack(self_l)).to(dev)
        edits_d = []
        if args.sparse_edits:                 # edits that turn grid k-1 into grid k (cyclically)
            for k in range(n_sets):
                e, i, m = synth.grid_edits(grids[k - 1], grids[k])
                edits_d.append(tuple(torch.from_numpy(a).to(dev) for a in (e, i, m)))
    else:
        cams_np = wl.cameras
        if cams_np.shape[0] < 8:
            # single-pose workloads: re-draw view angles so that every timed step renders new cameras
            rng = np.random.default_rng(synth.BASE_SEED + 100 + args.config)
            n_sets = 8
            cams_np = np.repeat(cams_np[:1], n_sets, axis=0).copy()
            cams_np[1:, :, 3] = rng.uniform(0, 2 * np.pi, size=cams_np[1:, :, 3].shape)
            cams_np[1:, :, 4] = rng.uniform(-np.pi / 6, np.pi / 6, size=cams_np[1:, :, 4].shape)
        n_sets = cams_np.shape[0]
        cams_d = torch.from_numpy(cams_np).to(dev)
        grids_d, self_d = [vox_d], None

    n, H, W = spec.num_obs, spec.height, spec.width
    rgb = torch.empty((n, H, W, 3), dtype=torch.uint8, device=dev)
    depth = torch.empty((n, H, W), dtype=torch.float32, device=dev)

    def step(i, ev=None):
        k = i % n_sets
        if args.sparse_edits and spec.dynamic and i > 0:
            batch.update_voxels(*edits_d[k], stream=stream)
        elif not args.static_worlds or i == 0:
            batch.upload_worlds(grids_d[k % len(grids_d)], pal_d, stream=stream)
        batch.set_cameras(cams_d[k], None if self_d is None else self_d[k], stream=stream)
        if ev is not None:
            ev[0].record()
        batch.render(rgb, depth, stream=stream)
        if ev is not None:
            ev[1].record()

    step(0)
    for i in range(args.warmup):
        step(i)
    events = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i, events[i])
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0

    render_ms = np.array([a.elapsed_time(b) for a, b in events])
    ms_per_step = elapsed * 1e3 / args.steps
    obs_per_s = n * args.steps / elapsed
    rays_per_obs = H * W
    alg_bytes = algorithmic_bytes_per_obs(spec) * n
    achieved = alg_bytes / (render_ms.mean() * 1e-3) / 1e9

    result = {
        "metric": "egocentric observations/sec (128\u00d772 RGB+depth) on 1 MI355X; % of HBM peak",
        "value": obs_per_s,
        "unit": "observations/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": spec.name, "num_envs": spec.num_envs, "agents_per_env": spec.agents_per_env,
                   "grid": list(spec.grid), "image": [W, H], "num_materials": spec.num_materials,
                   "observations_per_step": n, "camera_sets": int(n_sets),
                   "step": ("render only after one upload" if args.static_worlds else
                            "mv_update_voxels(device) + mv_set_cameras(device) + mv_render_batch"
                            if (args.sparse_edits and spec.dynamic) else
                            "mv_upload_worlds(device) + mv_set_cameras(device) + mv_render_batch")},
        "rays_per_s": obs_per_s * rays_per_obs,
        "render_kernel_ms": {"mean": float(render_ms.mean()), "median": float(np.median(render_ms)),
                             "p95": float(np.percentile(render_ms, 95))},
        "render_only_obs_per_s": n / (render_ms.mean() * 1e-3),
        "hbm_peak_fraction": achieved / HBM_PEAK_GBS,
        "generator_seconds": gen_s,
        "input_sha256": input_digest(wl),
    }
    traffic = measured_traffic(spec.name)
    mean_steps = ORACLE_MEAN_STEPS.get(args.config)
    alg_ops = algorithmic_lane_ops_per_ray(mean_steps) * rays_per_obs * n if mean_steps else None
    if alg_ops is not None:
        alu_achieved = alg_ops / (render_ms.mean() * 1e-3) / 1e9
        # plain vector arithmetic binds the render kernel (neither HBM nor LDS comes close, see below)
        result["roofline"] = {"bound": "alu", "kernel": "mv::render_kernel", "achieved": alu_achieved,
                              "peak": ALU_PEAK_GOPS, "unit": "G lane-instructions/s",
                              "frac": alu_achieved / ALU_PEAK_GOPS, "traffic": traffic,
                              "algorithmic_ops_per_launch": alg_ops, "oracle_mean_steps_per_ray": mean_steps}
        executed = measured_traffic(spec.name, 3)
        if executed is not None:
            # what the kernel really executes (profiled counter), next to the model's count
            result["roofline"]["executed_ops_per_launch"] = executed
            result["roofline"]["executed_frac"] = executed / (render_ms.mean() * 1e-3) / 1e9 / ALU_PEAK_GOPS
    result["hbm_roofline"] = {"bound": "hbm", "kernel": "mv::render_kernel", "achieved": achieved,
                              "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                              "traffic": traffic, "algorithmic_bytes_per_launch": alg_bytes,
                              "device_copy_GBs": device_copy_rate(torch)}
    lds_bytes = measured_traffic(spec.name, 2)
    if lds_bytes is not None:
        # LDS peak: 256 CUs x 128 bytes per clock x 2.4 GHz
        lds_peak = 256 * 128 * 2.4
        result["lds_roofline"] = {"bound": "lds", "kernel": "mv::render_kernel",
                                  "achieved": lds_bytes / (render_ms.mean() * 1e-3) / 1e9, "peak": lds_peak,
                                  "unit": "GB/s", "frac": lds_bytes / (render_ms.mean() * 1e-3) / 1e9 / lds_peak,
                                  "bytes_per_launch": lds_bytes}

    if not args.no_cpu_baseline:
        from oracle import oracle as orc
        cores = min(os.cpu_count() or 1, 16)
        envs = min(args.cpu_sample_envs, spec.num_envs)
        ob = orc.OracleBatch(envs, spec.agents_per_env, spec.grid, W, H, spec.num_materials)
        ob.upload_worlds(wl.voxels[:envs] if not spec.dynamic else grids[0][:envs], wl.palette[:envs])
        first_cams = (cams_l[0] if spec.dynamic else cams_np[0])[: envs * spec.agents_per_env]
        ob.set_cameras(first_cams, None if not spec.dynamic else self_l[0][: envs * spec.agents_per_env])
        # repeat whole passes (the same camera set: the oracle's cost does not depend on which) until the
        # sample amounts to roughly 10 s of CPU work
        passes, cpu_s = 0, 0.0
        t0 = time.perf_counter()
        while passes < 64 and cpu_s * cores < 10.0:
            ob.render(threads=cores, side_channels=False)
            passes += 1
            cpu_s = time.perf_counter() - t0
        steps_sample = ob.render(first_obs=0, count=min(64, envs * spec.agents_per_env), threads=cores).steps
        t1 = time.perf_counter()
        ob.render(first_obs=0, count=min(64, envs * spec.agents_per_env), threads=1, side_channels=False)
        one_core = min(64, envs * spec.agents_per_env) / (time.perf_counter() - t1)
        result["cpu_baseline"] = {"value": passes * envs * spec.agents_per_env / cpu_s, "unit": "observations/s",
                                  "cores": cores, "kind": "oracle",
                                  "sample": f"{passes} passes over the first {envs} environments "
                                            f"({envs * spec.agents_per_env} observations) of camera set 0, "
                                            f"{cpu_s:.2f} s wall on {cores} threads",
                                  "one_core_value": one_core,
                                  "mean_dda_steps_per_ray": float(steps_sample.mean())}
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
