"""The oracle's C sources under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only).

Every parity claim rests on oracle/mv_oracle.c and oracle/mv_definition.c, and their pins run on small
grids where a read past the end of the voxel or palette arrays could go unnoticed.  This test compiles both
files with -fsanitize=address,undefined (errors abort), and runs the whole pin file against that build in a
child interpreter that has the sanitizer runtime loaded first.  Nothing here touches the GPU or the HIP
library."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
ORACLE_DIR = os.path.join(ROOT, "oracle")


def _runtime(name):
    path = subprocess.run(["gcc", f"-print-file-name={name}"], check=True, capture_output=True, text=True).stdout.strip()
    return path if os.path.isabs(path) and os.path.exists(path) else None


def test_pins_pass_on_a_sanitized_build_of_the_oracle(tmp_path):
    asan = _runtime("libasan.so")
    if asan is None:
        pytest.skip("gcc has no AddressSanitizer runtime here")
    lib = tmp_path / "libmv_oracle_sanitized.so"
    subprocess.run(["gcc", "-std=c11", "-O1", "-g", "-fPIC", "-shared", "-ffp-contract=off", "-fno-fast-math",
                    "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer",
                    "-Wall", "-Wextra", "-o", str(lib), os.path.join(ORACLE_DIR, "mv_oracle.c"),
                    os.path.join(ORACLE_DIR, "mv_definition.c"), "-lm", "-lpthread"], check=True)
    env = dict(os.environ)
    # the sanitizer runtime must be the first library of the process; whatever is preloaded already stays
    env["LD_PRELOAD"] = " ".join(x for x in (asan, env.get("LD_PRELOAD", "")) if x)
    # Python itself is not leak-clean; the link-order check would object to other preloaded libraries
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=1"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env["MV_ORACLE_LIBRARY"] = str(lib)
    proc = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"), "-x", "-q",
                           "-p", "no:cacheprovider"], cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    tail = (proc.stdout + proc.stderr)[-3000:]
    assert proc.returncode == 0, tail
    assert " passed" in proc.stdout and "MV_ORACLE_LIBRARY" not in proc.stderr, tail
