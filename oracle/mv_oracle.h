/*
 * CPU oracle for the batched egocentric voxel-world render -- TEST INFRASTRUCTURE ONLY.
 *
 * This is a plain, slow, float64 implementation of what the GPU library computes.  It is used
 * by the test-suite, by the smoke check and by the benchmark's cpu_baseline leg, and by nothing
 * else: the product library never links, loads or calls it, and it shares no source with the
 * HIP code (own structs, own constants, own arithmetic).
 *
 * What is rendered follows the paper's problem statement (Sec. 3.2, Eq. 2: O = Render(S), one
 * observation per agent of every environment; App. A.2: 128x72 RGB observations; Sec. 4: flat
 * "monochrome" materials; Sec. 3: shading with simulated lighting).  The paper rasterises and
 * fixes no camera model, shading formula or depth output, so every numeric convention here is a
 * stated reading: pinhole camera (yaw about +z, pitch up-positive, no roll), the ray through
 * each pixel centre, the nearest solid voxel along it, Lambert + ambient shading of the entered
 * face, planar depth in voxel units.
 *
 * Two layers:
 *   - mv_definition.c : definition D, the nearest solid unit cube by testing the ray against
 *                       every solid voxel (slab test).  Obviously correct, O(voxels) per ray.
 *   - mv_oracle.c     : algorithm O, the 3D-DDA traversal (Amanatides-Woo style stepping) in
 *                       float64, pinned against D and against closed forms by tests/.
 *
 * Parity status: every function here is pinned (brute force, single-cube footprint, floor
 * depth, empty world, rotation/mirror/translation invariance, exhaustive quantisation).
 */
#ifndef MV_ORACLE_H
#define MV_ORACLE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MVO_FACE_INSIDE 6     /* ray origin lies inside a solid voxel            */
#define MVO_FACE_MISS   255   /* no solid voxel on the ray inside the grid        */

typedef struct mvo_batch mvo_batch;

typedef struct {
    int32_t num_envs, agents_per_env;
    int32_t grid_x, grid_y, grid_z;
    int32_t width, height;
    float   hfov_rad;
    int32_t num_materials;
    float   light_dir[3];     /* direction towards the light; normalised internally */
    float   ambient, diffuse;
    uint8_t sky_rgb[3];
    uint8_t pad_;
} mvo_config;

/* All pointers are host pointers.  Return 0 on success, -1 on a bad argument, -2 when called in
 * the wrong order (render before worlds and cameras are present), -3 on a range error. */
int  mvo_create(const mvo_config* cfg, mvo_batch** out);
void mvo_destroy(mvo_batch* b);
int  mvo_upload_worlds(mvo_batch* b, int32_t first_env, int32_t count,
                       const uint8_t* voxels /* [count,Z,Y,X] */,
                       const uint8_t* palette /* [count,M+1,3] or NULL = keep */);
/* Sparse edits of uploaded grids: voxel voxel_index[e] of environment env[e] becomes material[e]. */
int  mvo_update_voxels(mvo_batch* b, int32_t count, const int32_t* env, const int32_t* voxel_index,
                       const uint8_t* material);
int  mvo_set_cameras(mvo_batch* b, const float* cams /* [N*A,5] x,y,z,yaw,pitch */,
                     const int32_t* self_voxel /* [N*A] or NULL */);

/* Render observations first_obs .. first_obs+count-1.  Every output may be NULL.  Outputs are
 * indexed from the first rendered observation: rgb [count,H,W,3], the others [count,H,W]. */
int  mvo_render(mvo_batch* b, int32_t first_obs, int32_t count,
                uint8_t* rgb, float* depth, uint8_t* material, int32_t* hit_index, uint8_t* face,
                int32_t* steps, double* edge_margin, double* t_exact, int32_t num_threads);

/* Render single pixels (obs[i], row[i], col[i]); outputs are [n] (rgb [n,3]). */
int  mvo_render_pixels(mvo_batch* b, int64_t n, const int32_t* obs, const int32_t* row,
                       const int32_t* col, uint8_t* rgb, float* depth, uint8_t* material,
                       int32_t* hit_index, uint8_t* face, int32_t* steps, double* edge_margin,
                       double* t_exact);

/* Indicator bar over rendered colours: for each of the `count` observations starting at first_obs the
 * first floor(fraction*width + 0.5) columns (float32 arithmetic, clamped to 0..width) of the
 * width x height rectangle at (x, y) take fill_rgb, the others empty_rgb.  rgb is [count,H,W,3],
 * fraction [count].  active (may be NULL) is [N]: observations of environments with active == 0 are
 * left untouched. */
int  mvo_draw_bars(const mvo_batch* b, int32_t first_obs, int32_t count, uint8_t* rgb, const float* fraction,
                   int32_t x, int32_t y, int32_t width, int32_t height, const uint8_t fill_rgb[3],
                   const uint8_t empty_rgb[3], const uint8_t* active);

/* Overlay of geometric primitives (paper App. A.2: a pixel-space GUI of geometric primitives drawn over the
 * observation).  A primitive is an axis-aligned rectangle of pixels that lies inside the image.  Kind 0 paints it
 * in one colour.  Kinds 1 and 2 are gauges: with v = values[o * values_per_obs + value_index] and n =
 * floor(v * extent + 0.5) clamped to 0..extent (float32 product and sum, as for the bar), kind 1 paints the n
 * leftmost columns (extent = width) and kind 2 the n lowest rows (extent = height) in `rgb`, the rest of the
 * rectangle in `rest_rgb`.  The primitives are painted in list order: a later one covers an earlier one.
 * `rgb` holds `count` observations starting with observation first_obs.  Returns 0, -1 (argument) or -3 (range). */
typedef struct {
    int32_t x, y, width, height;
    uint8_t rgb[3];
    uint8_t kind;
    uint8_t rest_rgb[3];
    uint8_t value_index;
} mvo_rect;
int  mvo_draw_overlay(const mvo_batch* b, int32_t first_obs, int32_t count, uint8_t* rgb, const mvo_rect* rects,
                      int32_t num_rects, const float* values, int32_t values_per_obs, const uint8_t* active);

/* The 12-float camera record (P, F, R, U) of one observation and the float32 ray direction of
 * one pixel, exactly as the renderer uses them. */
int  mvo_camera_record(const mvo_batch* b, int32_t obs, float rec[12]);
int  mvo_pixel_ray(const mvo_batch* b, int32_t obs, int32_t row, int32_t col, float dir[3]);

/* The seven face intensities (six faces, then INSIDE) as float32. */
int  mvo_face_intensity(const mvo_batch* b, float out[7]);

/* Quantise one channel: palette value times intensity, rounded to the nearest integer in
 * float32 arithmetic, clamped to 255. */
uint8_t mvo_quantise(uint8_t palette_value, float intensity);

/* Definition D (mv_definition.c): nearest solid voxel along P + t*d, t >= 0, by testing every
 * solid voxel of one grid.  Returns 1 on a hit, 0 on a miss. */
int  mvd_first_hit(int32_t X, int32_t Y, int32_t Z, const uint8_t* vox,
                   const double P[3], const double d[3], int32_t self_voxel,
                   int32_t* hit_index, int32_t* face, double* t);
void mvd_first_hit_batch(int32_t X, int32_t Y, int32_t Z, const uint8_t* vox, int64_t n,
                         const double* P /* [n,3] */, const double* d /* [n,3] */,
                         const int32_t* self_voxel /* [n] or NULL */,
                         int32_t* hit_index, int32_t* face, double* t);

#ifdef __cplusplus
}
#endif
#endif
