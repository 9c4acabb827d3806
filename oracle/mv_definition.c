/*
 * Definition D of the CPU oracle: the nearest solid voxel along a ray, found by intersecting
 * the ray with the unit cube of EVERY solid voxel (slab test) and keeping the smallest entry
 * parameter t >= 0.  TEST INFRASTRUCTURE ONLY -- see mv_oracle.h.
 *
 * This is what "the first solid voxel the pixel ray meets" means, written out with no
 * traversal order at all; the DDA of mv_oracle.c must agree with it wherever the ray does not
 * pass exactly through a voxel edge.  Voxel (i,j,k) is the half-open cube
 * [i,i+1) x [j,j+1) x [k,k+1); faces are numbered by outward normal 0:-x 1:+x 2:-y 3:+y 4:-z
 * 5:+z, 6 = the origin itself lies inside the voxel.
 */
#include "mv_oracle.h"

#include <math.h>

int mvd_first_hit(int32_t X, int32_t Y, int32_t Z, const uint8_t* vox, const double P[3],
                  const double d[3], int32_t self_voxel, int32_t* hit_index, int32_t* face,
                  double* t)
{
    const int32_t self_hi = self_voxel >= 0 ? self_voxel + X * Y : -1;
    double best_t = INFINITY;
    int32_t best_idx = -1, best_face = MVO_FACE_MISS;

    for (int32_t k = 0; k < Z; ++k)
        for (int32_t j = 0; j < Y; ++j)
            for (int32_t i = 0; i < X; ++i) {
                const int32_t idx = (k * Y + j) * X + i;
                if (vox[idx] == 0 || idx == self_voxel || idx == self_hi) continue;
                const double lo[3] = { (double)i, (double)j, (double)k };

                int origin_inside = 1;
                for (int a = 0; a < 3; ++a)
                    if (P[a] < lo[a] || P[a] >= lo[a] + 1.0) origin_inside = 0;
                if (origin_inside) {
                    *hit_index = idx; *face = MVO_FACE_INSIDE; *t = 0.0;
                    return 1;
                }

                double t_enter = -INFINITY, t_leave = INFINITY;
                int enter_axis = -1, ok = 1;
                for (int a = 0; a < 3 && ok; ++a) {
                    if (d[a] == 0.0) {
                        if (P[a] < lo[a] || P[a] >= lo[a] + 1.0) ok = 0;
                        continue;
                    }
                    double t1 = (lo[a] - P[a]) / d[a];
                    double t2 = (lo[a] + 1.0 - P[a]) / d[a];
                    double tn = t1 < t2 ? t1 : t2, tf = t1 < t2 ? t2 : t1;
                    if (tn > t_enter) { t_enter = tn; enter_axis = a; }
                    if (tf < t_leave) t_leave = tf;
                }
                if (!ok || enter_axis < 0) continue;
                if (t_enter > t_leave || t_enter < 0.0) continue;
                if (t_enter < best_t) {
                    best_t = t_enter;
                    best_idx = idx;
                    best_face = 2 * enter_axis + (d[enter_axis] < 0.0 ? 1 : 0);
                }
            }
    if (best_idx < 0) return 0;
    *hit_index = best_idx; *face = best_face; *t = best_t;
    return 1;
}

void mvd_first_hit_batch(int32_t X, int32_t Y, int32_t Z, const uint8_t* vox, int64_t n,
                         const double* P, const double* d, const int32_t* self_voxel,
                         int32_t* hit_index, int32_t* face, double* t)
{
    for (int64_t r = 0; r < n; ++r) {
        int32_t hi = -1, fa = MVO_FACE_MISS;
        double tt = 0.0;
        if (!mvd_first_hit(X, Y, Z, vox, P + 3 * r, d + 3 * r, self_voxel ? self_voxel[r] : -1,
                           &hi, &fa, &tt)) {
            hi = -1; fa = MVO_FACE_MISS; tt = 0.0;
        }
        hit_index[r] = hi; face[r] = fa; t[r] = tt;
    }
}
