"""Writes profiles/oracle_mean_steps.txt: the mean number of per-cell DDA steps per ray of the CPU oracle on camera
set 0 of each benchmark workload (the S of the ALU roofline's "10*S + 60" lane-instructions per ray).  Calls only
the oracle and the seeded input generators.  The benchmark measures the same figure in its own oracle pass and
reads this file only when that pass is skipped.

    python -m tests.oracle_mean_steps [max_envs]
"""
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

from oracle import oracle as orc                       # noqa: E402
from paper_2107_08170_amd import synth                 # noqa: E402  (input generators only: no renderer arithmetic)


def mean_steps(index: int, max_envs: int) -> tuple:
    wl = synth.generate(index)
    s = wl.spec
    envs = min(max_envs, s.num_envs)
    obs = envs * s.agents_per_env
    ob = orc.OracleBatch(envs, s.agents_per_env, s.grid, s.width, s.height, s.num_materials)
    ob.upload_worlds(wl.voxels[:envs], wl.palette[:envs])
    ob.set_cameras(wl.cameras[0][:obs], None if wl.self_voxel is None else wl.self_voxel[0][:obs])
    total = 0
    for o0 in range(0, obs, 512):
        c = min(512, obs - o0)
        total += int(ob.render(first_obs=o0, count=c, threads=os.cpu_count() or 1, side_channels="steps").steps.sum(dtype=np.int64))
    return s.name, total / (obs * s.height * s.width), envs, obs


def main() -> int:
    max_envs = int(sys.argv[1]) if len(sys.argv) > 1 else 4096
    lines = ["# Mean per-cell DDA steps per ray of the CPU oracle, camera set 0 of each workload.",
             f"# Written by: python -m tests.oracle_mean_steps {max_envs}   (first <= {max_envs} environments of each workload)",
             "# workload  mean_steps_per_ray  environments  observations"]
    for index in (1, 2, 3, 4):
        name, mean, envs, obs = mean_steps(index, max_envs)
        lines.append(f"{name} {mean:.4f} {envs} {obs}")
        print(lines[-1], flush=True)
    with open(os.path.join(ROOT, "profiles", "oracle_mean_steps.txt"), "w") as f:
        f.write("\n".join(lines) + "\n")
    return 0


if __name__ == "__main__":
    sys.exit(main())
