"""The pins must notice plausible mistakes.  Each case plants one mistake in a COPY of the oracle's
source (a flipped sign, a swapped index, a transposed operand ...), compiles it on the CPU, runs the
pin battery of test_oracle_pins.py against the broken build and requires that at least one pin fails.
The unmodified build must pass the same battery.  Nothing here touches the GPU or the HIP library."""
import os
import shutil
import subprocess
import warnings

import numpy as np
import pytest

from tests import test_oracle_pins as pins

ORACLE_DIR = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "oracle")

# (name, file, text to find exactly once, replacement)
MISTAKES = [
    ("mirror image left-right", "mv_oracle.c", "(float)(2 * col + 1 - W) / (float)W", "(float)(W - 2 * col - 1) / (float)W"),
    ("flip image upside down", "mv_oracle.c", "(float)(H - 2 * row - 1) / (float)H", "(float)(2 * row + 1 - H) / (float)H"),
    ("sx divided by the height", "mv_oracle.c", "(float)(2 * col + 1 - W) / (float)W", "(float)(2 * col + 1 - W) / (float)H"),
    ("right vector negated", "mv_oracle.c", "double right[3] = { sy, -cy, 0.0 };", "double right[3] = { -sy, cy, 0.0 };"),
    ("up vector: horizontal part sign", "mv_oracle.c", "double up[3]    = { -sp * cy, -sp * sy, cp };",
     "double up[3]    = { sp * cy, sp * sy, cp };"),
    ("pitch sign", "mv_oracle.c", "double fwd[3]   = { cp * cy, cp * sy, sp };", "double fwd[3]   = { cp * cy, cp * sy, -sp };"),
    ("yaw measured from +y", "mv_oracle.c", "double fwd[3]   = { cp * cy, cp * sy, sp };", "double fwd[3]   = { cp * sy, cp * cy, sp };"),
    ("aspect ratio inverted", "mv_oracle.c", "b->tan_half_x * (double)cfg->height / (double)cfg->width",
     "b->tan_half_x * (double)cfg->width / (double)cfg->height"),
    ("up term dropped from the ray", "mv_oracle.c", "fmaf(sy, rec[9 + a], fmaf(sx, rec[6 + a], rec[3 + a]))",
     "fmaf(sx, rec[6 + a], rec[3 + a])"),
    ("R and U swapped in the ray", "mv_oracle.c", "fmaf(sy, rec[9 + a], fmaf(sx, rec[6 + a], rec[3 + a]))",
     "fmaf(sy, rec[6 + a], fmaf(sx, rec[9 + a], rec[3 + a]))"),
    ("next plane on the wrong side", "mv_oracle.c", "(double)(cell[axis] + (step[axis] > 0 ? 1 : 0))",
     "(double)(cell[axis] + (step[axis] > 0 ? 0 : 1))"),
    ("first plane on the wrong side", "mv_oracle.c", "t_max[a] = ((double)(cell[a] + 1) - P[a]) / d[a]; }",
     "t_max[a] = ((double)cell[a] - P[a]) / d[a]; }"),
    ("face parity swapped", "mv_oracle.c", "face = 2 * axis + (step[axis] < 0 ? 1 : 0);", "face = 2 * axis + (step[axis] > 0 ? 1 : 0);"),
    ("x and y swapped in the hit index", "mv_oracle.c",
     "        idx = (cell[2] * dim[1] + cell[1]) * dim[0] + cell[0];\n        found",
     "        idx = (cell[2] * dim[0] + cell[0]) * dim[1] + cell[1];\n        found"),
    ("z preferred at ties is fine, but y never chosen", "mv_oracle.c", "else if (t_max[1] <= t_max[2]) axis = 1;", "else if (0) axis = 1;"),
    ("euclidean instead of planar depth", "mv_oracle.c", "out->depth = (float)t_hit;",
     "out->depth = (float)(t_hit * sqrt(d[0] * d[0] + d[1] * d[1] + d[2] * d[2]));"),
    ("lit and unlit faces swapped", "mv_oracle.c", "double ndotl = (f & 1) ? L[f >> 1] : -L[f >> 1];",
     "double ndotl = (f & 1) ? -L[f >> 1] : L[f >> 1];"),
    ("light not normalised", "mv_oracle.c", "const double L[3] = { lx / ln, ly / ln, lz / ln };", "const double L[3] = { lx, ly, lz };"),
    ("colour truncated instead of rounded", "mv_oracle.c", "volatile float sum = prod + 0.5f;                          /* a second one        */",
     "volatile float sum = prod;"),
    ("own body is one voxel tall", "mv_oracle.c", "self_lo >= 0 ? self_lo + dim[0] * dim[1] : -1;", "-1;"),
    ("palette of environment 0 for everyone", "mv_oracle.c", "b->pal + (size_t)env * (size_t)(b->cfg.num_materials + 1) * 3;", "b->pal;"),
    ("agents share the first camera of the environment", "mv_oracle.c", "const float* rec = b->rec + 12 * (size_t)obs;\n    const double P[3]",
     "const float* rec = b->rec + 12 * (size_t)(obs - obs % b->cfg.agents_per_env);\n    const double P[3]"),
    ("clip against the wrong slab side", "mv_oracle.c", "double ta = ((d[a] > 0.0 ? 0.0 : (double)dim[a]) - P[a]) / d[a];",
     "double ta = ((d[a] > 0.0 ? (double)dim[a] : 0.0) - P[a]) / d[a];"),
    ("sky colour channels reversed", "mv_oracle.c", "out->rgb[0] = b->cfg.sky_rgb[0];", "out->rgb[0] = b->cfg.sky_rgb[2];"),
    ("bar width truncated", "mv_oracle.c", "volatile float sum = prod + 0.5f;\n        float cols", "volatile float sum = prod;\n        float cols"),
    ("overlay: primitives painted in reverse order", "mv_oracle.c", "const mvo_rect* q = &rects[k];\n            int32_t filled = 0;", "const mvo_rect* q = &rects[num_rects - 1 - k];\n            int32_t filled = 0;"),
    ("overlay: upward gauge fills from the top", "mv_oracle.c", "in_front = q->height - 1 - r < filled;", "in_front = r < filled;"),
    ("overlay: gauge length truncated", "mv_oracle.c", "volatile float sum = prod + 0.5f;\n                float n", "volatile float sum = prod;\n                float n"),
    ("overlay: upward gauge measured against the width", "mv_oracle.c", "const int32_t extent = q->kind == 1 ? q->width : q->height;", "const int32_t extent = q->width;"),
    ("overlay: gauge reads the first value column", "mv_oracle.c", "values[(size_t)o * values_per_obs + q->value_index]", "values[(size_t)o * values_per_obs]"),
    ("edits land one voxel further", "mv_oracle.c", "(size_t)voxel_index[e]] = material[e];", "(size_t)voxel_index[e] + 1] = material[e];"),
    ("margin: the crossing's own axis not skipped", "mv_oracle.c", "        if (a == axis) continue;\n        double q = P[a] + t * d[a];",
     "        double q = P[a] + t * d[a];"),
    ("margin: crossing point from the wrong direction component", "mv_oracle.c", "double q = P[a] + t * d[a];", "double q = P[a] + t * d[axis];"),
    ("margin: only the last crossing counts", "mv_oracle.c", "if (m < out->edge_margin) out->edge_margin = m;", "out->edge_margin = m;"),
    ("margin: the crossing into the grid forgotten", "mv_oracle.c", "out->edge_margin = crossing_margin(P, d, t0, entry_axis);", ""),
    ("margin: a ray that passes the whole grid by is never a tie", "mv_oracle.c", "out->edge_margin = worst;", ""),
    ("margin: passing by takes the smaller excess", "mv_oracle.c", "if (excess > worst) worst = excess;", "if (worst == 0.0 || excess < worst) worst = excess;"),
    ("step counter counts every other crossing", "mv_oracle.c", "out->steps += 1;", "out->steps += (cell[axis] & 1);"),
    ("brute force keeps the farthest voxel", "mv_definition.c", "if (t_enter < best_t) {", "if (best_idx < 0 || t_enter > best_t) {"),
    ("brute force ignores rays leaving the slab", "mv_definition.c", "if (t_enter > t_leave || t_enter < 0.0) continue;", "if (t_enter < 0.0) continue;"),
]


def _battery(orc):
    """Every pin of test_oracle_pins.py, with its parameters."""
    for seed in range(3):
        yield lambda s=seed: pins.test_dda_matches_definition_on_tiny_grids(orc, s)
    yield lambda: pins.test_definition_on_structured_world(orc)
    for row in pins._read_table("single_cube_footprint.txt"):
        yield lambda r=row: pins.test_single_cube_footprint_and_depth(orc, *r)
    for case in pins._FACE_CASES:
        yield lambda c=case: pins.test_six_faces_and_intensities(orc, *c)
    yield lambda: pins.test_face_intensity_table(orc)
    yield lambda: pins.test_off_axis_cube_pins_left_right_and_up_down(orc)
    yield lambda: pins.test_floor_depth_closed_form(orc)
    yield lambda: pins.test_pitched_camera_floor_landing_points(orc)
    yield lambda: pins.test_empty_world_is_sky(orc)
    yield lambda: pins.test_rotation_by_90_degrees_about_z(orc)
    yield lambda: pins.test_mirror_in_x_flips_the_image(orc)
    yield lambda: pins.test_integer_translation_inside_a_larger_grid(orc)
    yield lambda: pins.test_quantisation_exhaustive_vs_exact_rationals(orc)
    yield lambda: pins.test_observation_order_and_own_body(orc)
    yield lambda: pins.test_vertical_and_axis_parallel_rays_terminate(orc)
    yield lambda: pins.test_exact_zero_direction_components(orc)
    yield lambda: pins.test_sparse_edits_equal_a_fresh_upload(orc)
    yield lambda: pins.test_indicator_bar_closed_form(orc)
    yield lambda: pins.test_overlay_rectangles_paint_in_list_order(orc)
    yield lambda: pins.test_overlay_gauges_closed_form(orc)
    yield lambda: pins.test_edge_margin_flags_ties_at_the_grid_boundary(orc)
    yield lambda: pins.test_edge_margin_equals_plane_enumeration(orc)
    yield lambda: pins.test_edge_margin_flags_a_grazed_edge_inside_the_grid(orc)
    yield lambda: pins.test_edge_margin_flags_a_ray_that_passes_the_grid_by_at_its_rim(orc)
    yield lambda: pins.test_step_count_and_termination_bound(orc)
    yield lambda: pins.test_single_pixel_entry_point_equals_the_full_render(orc)


def _first_failure(orc):
    for run in _battery(orc):
        try:
            with warnings.catch_warnings():
                warnings.simplefilter("ignore")
                run()
        except (AssertionError, ValueError, IndexError, ZeroDivisionError) as exc:
            return exc
    return None


def _build_variant(tmp_path, file, old, new):
    work = tmp_path / "oracle_variant"
    work.mkdir()
    for name in ("mv_oracle.c", "mv_definition.c", "mv_oracle.h"):
        shutil.copy(os.path.join(ORACLE_DIR, name), work / name)
    text = (work / file).read_text()
    assert text.count(old) == 1, f"pattern must occur exactly once in {file}: {old!r} ({text.count(old)} found)"
    (work / file).write_text(text.replace(old, new))
    lib = work / "libvariant.so"
    subprocess.run(["gcc", "-std=c11", "-O1", "-fPIC", "-shared", "-ffp-contract=off", "-o", str(lib),
                    str(work / "mv_oracle.c"), str(work / "mv_definition.c"), "-lm", "-lpthread"], check=True,
                   capture_output=True)
    return str(lib)


def test_unmodified_oracle_passes_the_battery(orc):
    assert _first_failure(orc) is None


@pytest.mark.parametrize("name,file,old,new", MISTAKES, ids=[m[0] for m in MISTAKES])
def test_planted_mistake_is_caught(orc, tmp_path, name, file, old, new):
    lib = _build_variant(tmp_path, file, old, new)
    with orc.use_library(lib):
        failure = _first_failure(orc)
    assert failure is not None, f"no pin noticed the mistake: {name}"
