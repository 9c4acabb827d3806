#!/usr/bin/env python3
"""Benchmark of the batched egocentric render on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 2]

A step is one pass of the whole hot path over one batch of synthetic input that is already
resident in device memory: world upload + occupancy packing + colour tables (mv_upload_worlds),
camera records (mv_set_cameras, a fresh camera set every step) and the render
(mv_render_batch) of every observation.  Prints ONE JSON line: observations/s (whole job), the
roofline of the dominant kernel measured with HIP events around every render launch, and the CPU
oracle timed on a bounded sample of the same workload on the host cores.

Order of the run: all inputs are generated and copied to the device first; a "cold start" sample (the first 20
steps after that idle time) is taken; then the side measurements that use the GPU run: the other workloads, a
plain device copy, and the cameras + render protocol on the headline batch (100 steps).  The headline region (W
warm-up steps, K timed steps) follows them directly: a GPU that has been idle runs this kernel 10-25 % slower
for its first fifty to a hundred launches (about 25 ms), whatever the warm-up count, and the sustained rate is
what the metric asks for; the cold figure is reported next to it.  Delivery to host memory and the CPU oracle
come last.
"""
import argparse
import hashlib
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
LDS_PEAK_GBS = 256 * 128 * 2.4         # 256 CUs x 128 bytes per clock x 2.4 GHz
KERNEL_SOURCE = os.path.join(ROOT, "paper_2107_08170_amd", "csrc", "mv_kernels.hip")
TRAFFIC_PROFILE = os.path.join(ROOT, "profiles", "render_traffic.txt")
STEPS_PROFILE = os.path.join(ROOT, "profiles", "oracle_mean_steps.txt")


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


def kernel_source_sha256() -> str:
    with open(KERNEL_SOURCE, "rb") as f:
        return hashlib.sha256(f.read()).hexdigest()


def profiled_counters(workload: str):
    """Per-launch counter figures of the render kernel from the committed rocprofv3 summary: HBM bytes (FETCH_SIZE
    and WRITE_SIZE scaled against a plain copy), LDS bytes (from SQ_INSTS_LDS) and vector lane-instructions
    executed (SQ_INSTS_VALU x 64).  The summary names the SHA-256 of the kernel source it was measured on; when
    that is not the source of the library being timed, the figures are stale and nothing is returned."""
    try:
        with open(TRAFFIC_PROFILE) as f:
            lines = f.read().splitlines()
    except OSError:
        return None
    sha = next((ln.split()[-1] for ln in lines if ln.startswith("# kernel_source_sha256")), None)
    if sha != kernel_source_sha256():
        return None
    for ln in lines:
        parts = ln.split()
        if len(parts) >= 4 and parts[0] == workload:
            return {"hbm_bytes": float(parts[1]), "lds_bytes": float(parts[2]), "valu_lane_ops": float(parts[3]),
                    "kernel_source_sha256": sha}
    return None


def committed_mean_steps(workload: str):
    """Mean per-cell DDA steps per ray of the CPU oracle on camera set 0, from the committed summary written by
    ``python -m tests.oracle_mean_steps`` (used only when this run skips its own oracle pass)."""
    try:
        with open(STEPS_PROFILE) as f:
            for ln in f:
                parts = ln.split()
                if len(parts) >= 2 and parts[0] == workload:
                    return float(parts[1])
    except OSError:
        pass
    return None


def input_digest(wl) -> str:
    """SHA-256 over the generated grids, palettes and cameras: identifies the synthetic input of a run."""
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


class Leg:
    """One workload resident on the device: batch object, inputs of a few steps, output tensors."""

    def __init__(self, mv, synth, torch, np, wl, index, sparse_edits=False, tiles_per_block=0, coarse_level=0,
                 object_moves=False):
        spec = wl.spec
        dev = torch.device("cuda", 0)
        self.torch, self.np, self.spec, self.wl = torch, np, spec, wl
        self.stream = torch.cuda.current_stream().cuda_stream
        self.batch = mv.Batch(spec.num_envs, spec.agents_per_env, spec.grid, spec.num_materials, spec.width, spec.height,
                              tiles_per_block=tiles_per_block, coarse_level=coarse_level)
        self.pal_d = torch.from_numpy(wl.palette).to(dev)
        self.sparse = bool(sparse_edits and spec.dynamic)
        self.moves = bool(object_moves and spec.dynamic)
        self.edits_d, self.moves_d = [], []
        if spec.dynamic:
            # dynamic worlds: pre-compute the grids/cameras of a few steps on the host, keep them resident
            grids, cams_l, self_l = [wl.voxels], [wl.cameras[0]], [wl.self_voxel[0]]
            where = [synth.dynamic_positions(wl)]
            for _ in range(3):
                g, c, s = synth.dynamic_step(wl)
                grids.append(g); cams_l.append(c); self_l.append(s)
                where.append(synth.dynamic_positions(wl))
            self.grids_d = [torch.from_numpy(g).to(dev) for g in grids]
            self.cams_d = torch.from_numpy(np.stack(cams_l)).to(dev)
            self.self_d = torch.from_numpy(np.stack(self_l)).to(dev)
            self.first_grid, self.first_cams, self.first_self = grids[0], cams_l[0], self_l[0]
            if self.moves:                    # the objects' cells at step k-1 and at step k (cyclically)
                for k in range(len(grids)):
                    self.moves_d.append(tuple(torch.from_numpy(a).to(dev)
                                              for a in synth.object_moves(wl, where[k - 1], where[k])))
            if self.sparse:                   # edits that turn grid k-1 into grid k (cyclically)
                for k in range(len(grids)):
                    e, i, m = synth.grid_edits(grids[k - 1], grids[k])
                    self.edits_d.append(tuple(torch.from_numpy(a).to(dev) for a in (e, i, m)))
        else:
            cams_np = wl.cameras
            if cams_np.shape[0] < 8:
                # single-pose workloads: re-draw view angles so that every timed step renders new cameras
                rng = np.random.default_rng(synth.BASE_SEED + 100 + index)
                cams_np = np.repeat(cams_np[:1], 8, axis=0).copy()
                if index in (s.index for s in synth.EXTRA_SPECS.values()):
                    # these cameras are aimed (the outside ones at their arena): turn them a little only
                    cams_np[1:, :, 3] += rng.uniform(-0.3, 0.3, size=cams_np[1:, :, 3].shape)
                    cams_np[1:, :, 4] += rng.uniform(-0.1, 0.1, size=cams_np[1:, :, 4].shape)
                else:
                    cams_np[1:, :, 3] = rng.uniform(0, 2 * np.pi, size=cams_np[1:, :, 3].shape)
                    cams_np[1:, :, 4] = rng.uniform(-np.pi / 6, np.pi / 6, size=cams_np[1:, :, 4].shape)
            self.cams_d = torch.from_numpy(cams_np).to(dev)
            self.grids_d, self.self_d = [torch.from_numpy(wl.voxels).to(dev)], None
            self.first_grid, self.first_cams, self.first_self = wl.voxels, cams_np[0], None
        self.n_sets = int(self.cams_d.shape[0])
        n, H, W = spec.num_obs, spec.height, spec.width
        self.rgb = torch.empty((n, H, W, 3), dtype=torch.uint8, device=dev)
        self.depth = torch.empty((n, H, W), dtype=torch.float32, device=dev)

    borrow = False          # upload_worlds without the material copy (the batch reads the caller's device array)

    def step(self, i, ev=None, static_worlds=False, rgb=None, depth=None, stream=None):
        stream = self.stream if stream is None else stream
        k = i % self.n_sets
        if self.moves and i > 0:
            self.batch.move_voxels(*self.moves_d[k], stream=stream)
        elif self.sparse and i > 0:
            self.batch.update_voxels(*self.edits_d[k], stream=stream)
        elif not static_worlds or i == 0:
            self.batch.upload_worlds(self.grids_d[k % len(self.grids_d)], self.pal_d, stream=stream, borrow=self.borrow)
        self.batch.set_cameras(self.cams_d[k], None if self.self_d is None else self.self_d[k], stream=stream)
        if ev is not None:
            ev[0].record()
        self.batch.render(self.rgb if rgb is None else rgb, self.depth if depth is None else depth, stream=stream)
        if ev is not None:
            ev[1].record()

    def timed(self, steps, warmup, static_worlds=False):
        """`warmup` untimed steps, then exactly `steps` timed ones between two synchronisations; the render launch
        of every timed step is bracketed by events on the launch stream."""
        torch, np = self.torch, self.np
        self.step(0)
        for i in range(warmup):
            self.step(i, static_worlds=static_worlds)
        events = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            self.step(i if not static_worlds else i + 1, events[i], static_worlds=static_worlds)
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0
        render_ms = np.array([a.elapsed_time(b) for a, b in events])
        return elapsed, render_ms

    def step_name(self, static_worlds=False):
        if static_worlds:
            return "mv_set_cameras(device) + mv_render_batch (worlds uploaded once)"
        if self.moves:
            return "mv_move_voxels(device) + mv_set_cameras(device) + mv_render_batch"
        if self.sparse:
            return "mv_update_voxels(device) + mv_set_cameras(device) + mv_render_batch"
        return "mv_upload_worlds(device) + mv_set_cameras(device) + mv_render_batch"

    def close(self):
        self.batch.close()


def side_workload(mv, synth, torch, np, wl, index, steps=40, warmup=15, sparse_edits=False, object_moves=False):
    """obs/s, rays/s and render time of another workload under the same step definition (a shorter region)."""
    leg = Leg(mv, synth, torch, np, wl, index, sparse_edits=sparse_edits, object_moves=object_moves)
    elapsed, render_ms = leg.timed(steps, warmup)
    spec = wl.spec
    out = {"workload": spec.name, "grid": list(spec.grid), "image": [spec.width, spec.height],
           "observations_per_step": spec.num_obs, "step": leg.step_name(), "steps": steps, "warmup": warmup,
           "obs_per_s": spec.num_obs * steps / elapsed,
           "rays_per_s": spec.num_obs * steps / elapsed * spec.width * spec.height,
           "ms_per_step": elapsed * 1e3 / steps, "render_kernel_ms": float(render_ms.mean()),
           "render_hbm_fraction": algorithmic_bytes_per_obs(spec) * spec.num_obs / (render_ms.mean() * 1e-3) / 1e9
                                  / HBM_PEAK_GBS}
    leg.close()
    del leg
    torch.cuda.empty_cache()
    return out


def host_delivery(mv, torch, leg, steps=12):
    """Observations/s that reach host memory: the step runs on one stream into one of two sets of output tensors
    while the previous step's observations are copied to pinned host memory on a second stream
    (mv_fetch_observations), the way a CPU consumer would be fed."""
    spec = leg.spec
    n, H, W = spec.num_obs, spec.height, spec.width
    rgb2, depth2 = torch.empty_like(leg.rgb), torch.empty_like(leg.depth)
    outs = [(leg.rgb, leg.depth), (rgb2, depth2)]
    pinned = [(mv.PinnedBuffer(n * H * W * 3), mv.PinnedBuffer(n * H * W * 4)) for _ in range(2)]
    compute, copy = torch.cuda.Stream(), torch.cuda.Stream()
    rendered = [torch.cuda.Event() for _ in range(2)]
    copied = [torch.cuda.Event() for _ in range(2)]
    torch.cuda.synchronize()

    def one(i):
        b = i % 2
        compute.wait_event(copied[b])                      # the buffer's last copy has left it
        leg.step(i, rgb=outs[b][0], depth=outs[b][1], stream=compute.cuda_stream)
        rendered[b].record(compute)
        copy.wait_event(rendered[b])
        leg.batch.fetch_observations(outs[b][0], outs[b][1], 0, n, pinned[b][0].address, pinned[b][1].address,
                                     stream=copy.cuda_stream)
        copied[b].record(copy)

    for b in range(2):
        copied[b].record(copy)
    for i in range(3):
        one(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        one(i)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    for pr, pd in pinned:
        pr.close(); pd.close()
    bytes_per_step = n * H * W * 7
    return {"obs_per_s": n * steps / elapsed, "ms_per_step": elapsed * 1e3 / steps, "steps": steps,
            "device_to_host_GBs": bytes_per_step * steps / elapsed / 1e9,
            "protocol": "mv_upload_worlds + mv_set_cameras + mv_render_batch on one stream, mv_fetch_observations of "
                        "all observations (colour + depth) into pinned host memory on a second stream, two sets of "
                        "output tensors"}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    # defaults: long enough to average launch-to-launch variation out; the whole timed region still lasts well
    # under a second
    ap.add_argument("--steps", type=int, default=500)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--config", type=int, default=2, help="workload index 1..4 (default 2: 4096 envs x 2 agents)")
    ap.add_argument("--tiles-per-block", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-envs", type=int, default=4096)
    ap.add_argument("--static-worlds", action="store_true",
                    help="headline region with the worlds uploaded once instead of every step (not the headline number)")
    ap.add_argument("--sparse-edits", action="store_true",
                    help="dynamic workload only: send the changed voxels of each step with mv_update_voxels instead "
                         "of re-uploading whole grids")
    ap.add_argument("--coarse-level", type=int, default=0,
                    help="1: render with the optional second occupancy level (same images; measured slower)")
    ap.add_argument("--no-other-workloads", action="store_true",
                    help="skip the side measurements on the other workloads (profiling runs)")
    ap.add_argument("--no-host-delivery", action="store_true", help="skip the delivery-to-host-memory measurement")
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

    # ---- inputs: everything is generated before the GPU is asked for anything
    spec = synth.SPECS[args.config]
    t0 = time.time()
    wl = synth.generate(args.config)
    gen_s = time.time() - t0
    with_others = args.config == 2 and not args.no_other_workloads and not args.static_worlds and not args.sparse_edits
    others = []
    if with_others:
        others = [(c, synth.generate(c), "upload") for c in (1, 3, 4)]
        others.insert(2, (3, synth.generate(3), "edits"))
        others.insert(3, (3, synth.generate(3), "moves"))
        others += [(s.index, synth.generate_extra(name), "upload") for name, s in synth.EXTRA_SPECS.items()]
    leg = Leg(mv, synth, torch, np, wl, args.config, sparse_edits=args.sparse_edits, tiles_per_block=args.tiles_per_block,
              coarse_level=args.coarse_level)
    n, H, W = spec.num_obs, spec.height, spec.width

    # ---- the first steps after the idle time of the set-up, for the record
    cold_el, cold_rm = leg.timed(20, 0)

    # ---- side measurements that keep the GPU busy right up to the headline region
    other_results = []
    for index, other_wl, how in others:
        other_results.append(side_workload(mv, synth, torch, np, other_wl, index, sparse_edits=how == "edits",
                                           object_moves=how == "moves"))
        del other_wl
    others = []
    copy_rate = device_copy_rate(torch)
    # a GPU that has been idle runs the render kernel 10-25 % slower for its first fifty to a hundred launches: a
    # hundred steps of the cameras + render protocol, not reported, take it out of that state
    if not args.static_worlds and not args.sparse_edits:
        leg.timed(100, 10, static_worlds=True)

    # ---- headline: W warm-up steps, K timed steps
    elapsed, render_ms = leg.timed(args.steps, args.warmup, static_worlds=args.static_worlds)
    # the cameras + render protocol (worlds uploaded once), a fixed 100 steps straight after the headline region
    static_result = None
    if not args.static_worlds and not args.sparse_edits:
        el2, rm2 = leg.timed(100, 10, static_worlds=True)
        static_result = {"step": leg.step_name(True), "steps": 100, "warmup": 10, "obs_per_s": n * 100 / el2,
                         "ms_per_step": el2 * 1e3 / 100, "render_kernel_ms": float(rm2.mean())}
    # the headline step with borrowed worlds (bit rows re-packed every step from the caller's device array, no
    # material copy), a fixed 100 steps; ends with a copying upload so that what follows sees the batch as before
    borrowed_result = None
    if not args.static_worlds and not args.sparse_edits:
        leg.borrow = True
        el3, rm3 = leg.timed(100, 10)
        leg.borrow = False
        leg.step(0)
        borrowed_result = {"step": "mv_upload_worlds(device, borrowed: no material copy) + mv_set_cameras(device) + "
                                   "mv_render_batch", "steps": 100, "warmup": 10, "obs_per_s": n * 100 / el3,
                           "ms_per_step": el3 * 1e3 / 100, "render_kernel_ms": float(rm3.mean())}
    ms_per_step = elapsed * 1e3 / args.steps
    obs_per_s = n * args.steps / elapsed
    rays_per_obs = H * W
    alg_bytes = algorithmic_bytes_per_obs(spec) * n
    achieved = alg_bytes / (render_ms.mean() * 1e-3) / 1e9

    result = {
        "metric": "egocentric observations/sec (128×72 RGB+depth) on 1 MI355X; % of HBM peak",
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
                   "observations_per_step": n, "camera_sets": int(leg.n_sets),
                   "step": leg.step_name(args.static_worlds), "coarse_level": args.coarse_level},
        "rays_per_s": obs_per_s * rays_per_obs,
        "render_kernel_ms": {"mean": float(render_ms.mean()), "median": float(np.median(render_ms)),
                             "p95": float(np.percentile(render_ms, 95))},
        "render_only_obs_per_s": n / (render_ms.mean() * 1e-3),
        "hbm_peak_fraction": achieved / HBM_PEAK_GBS,
        "generator_seconds": gen_s,
        "input_sha256": input_digest(wl),
        "run_order": "inputs generated and uploaded; cold-start sample; other workloads; device copy; 110 unreported "
                     "steps of the cameras+render protocol; headline region; cameras+render protocol (100 steps); "
                     "borrowed-worlds step (100 steps); delivery to host; CPU oracle",
        "cold_start": {"what": "the first 20 steps after the set-up's idle time, no warm-up",
                       "obs_per_s": n * 20 / cold_el, "ms_per_step": cold_el * 1e3 / 20,
                       "render_kernel_ms": float(cold_rm.mean())},
    }
    if with_others:
        result["other_workloads"] = other_results

    if static_result is not None:
        result["static_worlds_obs_per_s"] = static_result["obs_per_s"]
        result["static_worlds"] = static_result
    if borrowed_result is not None:
        result["borrowed_worlds"] = borrowed_result
    if not args.no_host_delivery and not spec.dynamic:
        result["delivered_to_host"] = host_delivery(mv, torch, leg)

    # ---- the oracle on the host cores: bounded sample of the same workload; also the per-ray step count that
    #      the ALU roofline is priced with
    mean_steps, steps_source = None, None
    if not args.no_cpu_baseline:
        from oracle import oracle as orc
        cores = min(os.cpu_count() or 1, 16)
        envs = min(args.cpu_sample_envs, spec.num_envs)
        obs = envs * spec.agents_per_env
        ob = orc.OracleBatch(envs, spec.agents_per_env, spec.grid, W, H, spec.num_materials)
        ob.upload_worlds(leg.first_grid[:envs], wl.palette[:envs])
        ob.set_cameras(leg.first_cams[:obs], None if leg.first_self is None else leg.first_self[:obs])
        # repeat whole passes (the same camera set: the oracle's cost does not depend on which) until the
        # sample amounts to roughly 10 s of CPU work
        passes, cpu_s = 0, 0.0
        t0 = time.perf_counter()
        while passes < 64 and cpu_s * cores < 10.0:
            ob.render(threads=cores, side_channels=False)
            passes += 1
            cpu_s = time.perf_counter() - t0
        # one more pass over the same observations for the step counter, in chunks that keep the arrays small
        total_steps, chunk = 0, 1024
        for o0 in range(0, obs, chunk):
            c = min(chunk, obs - o0)
            total_steps += int(ob.render(first_obs=o0, count=c, threads=cores, side_channels="steps").steps.sum(dtype=np.int64))
        mean_steps = total_steps / (obs * H * W)
        steps_source = f"this run's oracle pass over {obs} observations of camera set 0"
        t1 = time.perf_counter()
        ob.render(first_obs=0, count=min(64, obs), threads=1, side_channels=False)
        one_core = min(64, obs) / (time.perf_counter() - t1)
        result["cpu_baseline"] = {"value": passes * obs / cpu_s, "unit": "observations/s",
                                  "cores": cores, "kind": "oracle",
                                  "sample": f"{passes} passes over the first {envs} environments "
                                            f"({obs} observations) of camera set 0, "
                                            f"{cpu_s:.2f} s wall on {cores} threads",
                                  "one_core_value": one_core,
                                  "mean_dda_steps_per_ray": mean_steps}
    else:
        mean_steps = committed_mean_steps(spec.name)
        steps_source = "profiles/oracle_mean_steps.txt" if mean_steps is not None else None

    # ---- rooflines of the render kernel (the dominant kernel), all priced with this run's mean launch time
    launch_s = render_ms.mean() * 1e-3
    prof = profiled_counters(spec.name)
    traffic = prof["hbm_bytes"] if prof else None
    if mean_steps is not None:
        alg_ops = algorithmic_lane_ops_per_ray(mean_steps) * rays_per_obs * n
        alu_achieved = alg_ops / launch_s / 1e9
        # plain vector arithmetic binds the render kernel (neither HBM nor LDS comes close, see below)
        result["roofline"] = {"bound": "alu", "kernel": "mv::render_kernel", "achieved": alu_achieved,
                              "peak": ALU_PEAK_GOPS, "unit": "G lane-instructions/s",
                              "frac": alu_achieved / ALU_PEAK_GOPS, "traffic": traffic,
                              "algorithmic_ops_per_launch": alg_ops, "oracle_mean_steps_per_ray": mean_steps,
                              "mean_steps_source": steps_source}
        if prof:
            # what the kernel really executes (profiled counter), next to the model's count
            result["roofline"]["executed_ops_per_launch"] = prof["valu_lane_ops"]
            result["roofline"]["executed_frac"] = prof["valu_lane_ops"] / launch_s / 1e9 / ALU_PEAK_GOPS
    result["hbm_roofline"] = {"bound": "hbm", "kernel": "mv::render_kernel", "achieved": achieved,
                              "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                              "traffic": traffic, "algorithmic_bytes_per_launch": alg_bytes,
                              "device_copy_GBs": copy_rate}
    if prof:
        result["lds_roofline"] = {"bound": "lds", "kernel": "mv::render_kernel",
                                  "achieved": prof["lds_bytes"] / launch_s / 1e9, "peak": LDS_PEAK_GBS,
                                  "unit": "GB/s", "frac": prof["lds_bytes"] / launch_s / 1e9 / LDS_PEAK_GBS,
                                  "bytes_per_launch": prof["lds_bytes"]}
        result["from_profile"] = {"file": "profiles/render_traffic.txt",
                                  "fields": ["roofline.traffic", "roofline.executed_ops_per_launch",
                                             "hbm_roofline.traffic", "lds_roofline.bytes_per_launch"],
                                  "kernel_source_sha256": prof["kernel_source_sha256"]}
    else:
        result["from_profile"] = None          # no counter summary for this kernel source: those fields are left out
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
