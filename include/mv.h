/*
 * mv.h -- C ABI of the batched egocentric voxel-world renderer for AMD MI355X (gfx950).
 *
 * One batch object holds N independent environments, each a voxel grid with one material id per
 * voxel, and A agent cameras per environment (paper Sec. 3.2: one simulator instance hosts N
 * environments with M agents each; here A = M).  One call renders the observation of every agent
 * of every environment in a single GPU request (paper Sec. 3.2, Eq. 2: O = Render(S)), as an
 * [N*A, H, W, 3] uint8 colour tensor (paper App. A.2: 128x72 RGB observations) plus an
 * [N*A, H, W] float32 depth tensor, both left in device memory (paper Sec. 3.2, last paragraph:
 * observations may stay on the GPU).  Observation index = env * A + agent (paper App. A.1: a
 * vector of N x M observations).
 *
 * What a pixel holds (the paper rasterises and gives no formula; this is the stated reading):
 * the ray from the camera position through the pixel centre of a pinhole camera (yaw about +z
 * measured from +x, pitch positive upwards, no roll, horizontal field of view hfov, square
 * pixels, row 0 at the top, column 0 at the left) is followed voxel by voxel (3D DDA) to the
 * first solid voxel (material id != 0) that is not part of the camera's own body.  Colour is that
 * voxel's palette colour (paper Sec. 4: flat "monochrome" materials, re-drawn per episode, hence
 * one palette per environment) times ambient + diffuse * max(0, n.L) for the face the ray entered
 * through, rounded to nearest; depth is the planar distance along the camera's forward axis in
 * voxel units.  Rays that leave the grid get sky_rgb and depth 0.
 *
 * Coordinates: voxel (i,j,k) is the cube [i,i+1) x [j,j+1) x [k,k+1), z is up, unit voxels.
 * Grids are stored x fastest: linear voxel index = (k*Y + j)*X + i.
 *
 * All entry points return MV_OK (0) or a negative mv_status; none throws, aborts or prints.
 * mv_last_error() returns a thread-local, NUL-terminated description of the last failure on
 * the calling thread.  Work is enqueued on the caller's HIP stream and the calls return without
 * synchronising; ordering between calls is stream order.  A batch must not be used from two
 * threads at once, and calls that touch the same batch from different streams must be ordered
 * by the caller (events or synchronisation): the batch's device buffers carry no locks.  Calls
 * that take host memory (src_is_device == 0) validate it, copy it and wait for the copy, so
 * they return only when the stream has passed them; the device-memory forms never wait and
 * allocate nothing, which makes a step built from them capturable in a HIP graph.
 */
#ifndef MV_H
#define MV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    MV_OK           =  0,
    MV_ERR_ARG      = -1,   /* null pointer, non-positive size, non-finite camera (host data)      */
    MV_ERR_STATE    = -2,   /* render before every environment and the cameras have been supplied  */
    MV_ERR_RANGE    = -3,   /* environment range outside the batch, material id > num_materials    */
    MV_ERR_CAPACITY = -4,   /* grid + image tile do not fit the per-workgroup LDS plan             */
    MV_ERR_HIP      = -5    /* a HIP runtime call failed; text in mv_last_error()                  */
} mv_status;

/* Face codes written to aux_face: outward normal of the voxel face the ray entered through. */
#define MV_FACE_NEG_X   0
#define MV_FACE_POS_X   1
#define MV_FACE_NEG_Y   2
#define MV_FACE_POS_Y   3
#define MV_FACE_NEG_Z   4
#define MV_FACE_POS_Z   5
#define MV_FACE_INSIDE  6     /* camera position is inside a solid voxel: depth 0, ambient only */
#define MV_FACE_MISS    255

typedef struct mv_batch mv_batch;     /* opaque; created and destroyed by the library */

typedef struct {
    int32_t num_envs;          /* N >= 1                                                          */
    int32_t agents_per_env;    /* A >= 1                                                          */
    int32_t grid_x, grid_y, grid_z;   /* voxels per axis, each >= 1                               */
    int32_t width, height;     /* image size in pixels, each >= 1 (128x72 in the paper)           */
    float   hfov_rad;          /* horizontal field of view, 0 < hfov < pi                         */
    int32_t num_materials;     /* 1..255; id 0 means empty                                        */
    float   light_dir[3];      /* direction TOWARDS the light, any non-zero length                */
    float   ambient, diffuse;  /* face intensity = ambient + diffuse * max(0, n.L)                */
    uint8_t sky_rgb[3];        /* colour of rays that leave the grid                              */
    uint8_t coarse_level;      /* 0 (default) or 1: 1 adds a second, coarser occupancy level (the OR of
                                  pairs of grid rows) that long rays use to cross empty space in fewer
                                  steps; results are the same bit for bit; grids up to 64x64 only      */
    int32_t device;            /* HIP device ordinal                                              */
    int32_t tiles_per_block;   /* 0 = choose automatically; otherwise the number of 8x8-pixel
                                  tiles one workgroup renders (a launch-shape knob, results do
                                  not depend on it)                                               */
} mv_config;

/* Fill *cfg with the defaults used throughout the paper-shaped workloads: 128x72 pixels, hfov
 * pi/2, light towards (1,2,3), ambient 0.30, diffuse 0.70, sky (135,206,235), device 0; the
 * sizes (num_envs, agents_per_env, grid, num_materials) are set to 0 and must be filled in. */
void mv_default_config(mv_config* cfg);

/* Create a batch on cfg->device (paper Sec. 3.2: N environments x M agents per instance).
 * Allocates all device memory the batch will ever use: material grids N*X*Y*Z bytes,
 * occupancy bits, per-environment shaded colour tables, camera records.  *out is written only
 * on success.  Grids up to 64x64 voxels in x and y take the fast row-scan traversal; wider grids
 * are rendered with a plain per-cell DDA.  Errors: MV_ERR_ARG (bad field), MV_ERR_CAPACITY (the
 * occupancy bits of one grid do not fit in the 160 KiB of LDS of a compute unit), MV_ERR_HIP. */
int mv_create_batch(const mv_config* cfg, mv_batch** out);

/* Replace the voxel grids of environments first_env .. first_env+count-1 (paper Sec. 3.1: the
 * world is a voxel grid; Sec. 4: layouts and materials are randomised per episode).
 *   voxels  : [count, Z, Y, X] uint8 material ids, x fastest.  Host memory if src_is_device == 0,
 *             device memory on the batch's device otherwise.  Copied; the caller keeps ownership
 *             and may reuse the buffer once the stream has passed this call (host memory: on
 *             return).
 *   palette : [count, num_materials+1, 3] uint8 RGB, row 0 ignored; same memory space as voxels;
 *             NULL keeps the palettes already uploaded.
 * Packs occupancy bits and re-shades the colour tables on `stream`.  Host data is validated
 * (material id > num_materials -> MV_ERR_RANGE, nothing is changed); device data is not, ids
 * above num_materials are clamped to num_materials when shading.
 * src_is_device == MV_SRC_DEVICE_BORROWED (a simulator that keeps its worlds on the GPU, paper Sec. 3.2): the
 * material ids are NOT copied.  The call must name every environment (first_env 0, count N); the occupancy
 * bits are packed from the caller's array, and every render up to the next mv_upload_worlds reads the material
 * of a hit voxel from that array, which the caller keeps alive and does not change meanwhile (to change it, change it
 * and call again: that re-packs, still without a copy).  While the batch borrows, mv_update_voxels, mv_move_voxels,
 * the edits of mv_step and uploads of part of the environments return MV_ERR_STATE; an upload of all environments
 * with src_is_device 0 or 1 ends the borrowing.  The palette is copied as always.
 * Errors: MV_ERR_ARG, MV_ERR_RANGE, MV_ERR_STATE, MV_ERR_HIP. */
#define MV_SRC_DEVICE_BORROWED 2
int mv_upload_worlds(mv_batch* batch, int32_t first_env, int32_t count, const uint8_t* voxels,
                     const uint8_t* palette, int32_t src_is_device, void* hip_stream);

/* Change single voxels of worlds that are already uploaded (paper Sec. 3.1-3.2: agents move boxes
 * and themselves through the voxel grid at every physics step; the state S changes a little per
 * step, not wholesale).  Edit e sets voxel voxel_index[e] (linear index (k*Y+j)*X+i) of environment
 * env[e] to material[e]; 0 empties the voxel.
 *   env, voxel_index : [count] int32;  material : [count] uint8.  All three in host memory if
 *   src_is_device == 0 (validated: MV_ERR_RANGE for an environment, index or material id out of range,
 *   nothing is changed), else in device memory (not validated; out-of-range edits are dropped).
 * Within one call every edit that empties a voxel (material 0) is applied before every edit that fills one,
 * whatever their order in the list: an object may move into the voxel another one leaves in the same step.
 * Two fills of the same voxel in one call are not ordered (either material may win).
 * The occupancy bit rows are patched in place with atomics; the per-environment "highest solid layer"
 * bound only grows (it stays a valid bound when the top voxel is removed).  count == 0 is a no-op.
 * Errors: MV_ERR_ARG, MV_ERR_RANGE, MV_ERR_STATE (an addressed environment has no grid yet; host data
 * only), MV_ERR_HIP. */
int mv_update_voxels(mv_batch* batch, int32_t count, const int32_t* env, const int32_t* voxel_index,
                     const uint8_t* material, int32_t src_is_device, void* hip_stream);

/* Re-stamp objects that moved, from their positions (paper Sec. 3.1-3.2: agents push boxes around and move
 * themselves; an object occupies whole voxels, an agent's body two of them).  Entry e says that one voxel of an
 * object of environment env[e] was at from_voxel[e] and is now at to_voxel[e] (linear indices; -1 = nowhere: the
 * object appears or disappears) and has material[e] (1..num_materials; 0 = nothing to draw).  Every `from` voxel
 * of the call is emptied first, then every `to` voxel is filled, so objects may swap places, follow each other or
 * stay where they are (from == to) in one call; two objects must not end in the same voxel.  The same as
 * mv_update_voxels with one clearing and one filling edit per entry, without the caller building those lists.
 *   env, from_voxel, to_voxel : [count] int32;  material : [count] uint8; host memory if src_is_device == 0
 *   (validated: MV_ERR_RANGE, MV_ERR_STATE as for mv_update_voxels, nothing is changed), else device memory (not
 *   validated; out-of-range entries are skipped).
 * Errors: MV_ERR_ARG, MV_ERR_RANGE, MV_ERR_STATE, MV_ERR_HIP. */
int mv_move_voxels(mv_batch* batch, int32_t count, const int32_t* env, const int32_t* from_voxel,
                   const int32_t* to_voxel, const uint8_t* material, int32_t src_is_device, void* hip_stream);

/* Set all N*A cameras (paper Sec. 3.2: cameras are entities of the state S that Render reads).
 *   cams       : [N*A, 5] float32 rows (x, y, z, yaw, pitch), observation order env*A+agent.
 *   self_voxel : [N*A] int32, linear index of the LOWER voxel of the camera's own 1x1x2 body
 *                (that voxel and the one directly above are invisible to this camera only), or
 *                -1 for none; NULL means -1 everywhere.
 * Host memory if src_is_device == 0 (validated: non-finite value -> MV_ERR_ARG), else device
 * memory (not validated).  The camera basis is computed on the GPU in float64 and rounded to
 * float32 records on `stream`.  Errors: MV_ERR_ARG, MV_ERR_RANGE (a self_voxel outside the grid; host data
 * only), MV_ERR_HIP. */
int mv_set_cameras(mv_batch* batch, const float* cams, const int32_t* self_voxel,
                   int32_t src_is_device, void* hip_stream);

/* Render every observation (paper Sec. 3.2, Eq. 2) into caller-owned DEVICE memory:
 *   rgb           : [N*A, H, W, 3] uint8, required.
 *   depth         : [N*A, H, W] float32, required; 0.0f where the ray leaves the grid.
 *   aux_material  : [N*A, H, W] uint8 material id of the hit voxel (0 on a miss), or NULL.
 *   aux_hit_index : [N*A, H, W] int32 linear index of the hit voxel (-1 on a miss), or NULL.
 *   aux_face      : [N*A, H, W] uint8 MV_FACE_* code, or NULL.
 * One kernel launch on `stream`; returns without synchronising.  The kernel keeps the lowest layers of each
 * grid on chip, as many as the tallest world uploaded so far needs (learnt from earlier kernels without
 * synchronising); the first launch after taller worlds arrive renders them through device memory (slower,
 * same accuracy, not necessarily the same bits at exact ties), later launches adapt.  While `stream` is being
 * captured into a HIP graph that choice would be frozen into the graph, so a captured launch keeps ALL layers
 * on chip instead (a few per cent slower than the adaptive choice on low worlds, never the slow path on a
 * replay over taller ones); a caller who knows the tallest world the graph will ever see can fix a smaller
 * number with mv_debug_set_staged_layers before capturing.
 * Errors: MV_ERR_ARG, MV_ERR_STATE (some environment or the cameras never supplied), MV_ERR_HIP. */
int mv_render_batch(mv_batch* batch, uint8_t* rgb, float* depth, uint8_t* aux_material,
                    int32_t* aux_hit_index, uint8_t* aux_face, void* hip_stream);

/* Choose which environments the next renders draw (paper App. A.1: environments reset on their own
 * and the last observation of a finished episode is never synthesised).
 *   active : [N] uint8, non-zero = render this environment's A observations; NULL = all (default).
 * Host memory if src_is_device == 0, else device memory; copied on `stream`.  Observations of inactive
 * environments are not touched by mv_render_batch (whatever the caller's tensors held stays there).
 * Errors: MV_ERR_ARG, MV_ERR_HIP. */
int mv_set_active(mv_batch* batch, const uint8_t* active, int32_t src_is_device, void* hip_stream);

/* A horizontal indicator bar drawn over every observation (paper App. A.2: a pixel-space GUI of
 * geometric primitives, used to show the agents the time left in the episode). */
typedef struct {
    int32_t x, y;              /* top-left pixel of the bar                                        */
    int32_t width, height;     /* in pixels; the bar must lie inside the image                     */
    uint8_t fill_rgb[3];       /* colour of the filled part (the left fraction of the bar)         */
    uint8_t empty_rgb[3];      /* colour of the rest of the bar                                    */
    uint8_t reserved[2];       /* must be 0                                                        */
} mv_bar;

/* Draw the bar into an already rendered colour tensor, in place, after the render on `stream`.
 *   rgb      : device [N*A, H, W, 3] uint8 (the tensor given to mv_render_batch).
 *   fraction : [N*A] float32, the filled share of each observation's bar; host memory if
 *              src_is_device == 0 (validated: non-finite -> MV_ERR_ARG), else device memory.
 * The first floor(fraction*width + 0.5) columns of the bar (float32 arithmetic, clamped to
 * 0..width) take fill_rgb, the others empty_rgb.  Depth is not touched.  Inactive environments
 * (mv_set_active) are skipped.  Errors: MV_ERR_ARG (null, bar outside the image), MV_ERR_HIP. */
int mv_draw_bars(mv_batch* batch, uint8_t* rgb, const float* fraction, const mv_bar* bar,
                 int32_t src_is_device, void* hip_stream);

/* An overlay of geometric primitives drawn over every observation (paper App. A.2: the pixel-space GUI is made of
 * geometric primitives).  A primitive is an axis-aligned rectangle of pixels that must lie inside the image. */
#define MV_MAX_OVERLAY_RECTS  32
#define MV_MAX_OVERLAY_VALUES 8
enum {
    MV_RECT_SOLID       = 0,    /* the whole rectangle in `rgb`                                            */
    MV_RECT_GAUGE_RIGHT = 1,    /* the n leftmost columns in `rgb`, the others in `rest_rgb`               */
    MV_RECT_GAUGE_UP    = 2     /* the n lowest rows in `rgb`, the others in `rest_rgb`                     */
};
typedef struct {
    int32_t x, y;              /* top-left pixel                                                          */
    int32_t width, height;     /* in pixels                                                               */
    uint8_t rgb[3];            /* colour of the rectangle, or of the filled part of a gauge               */
    uint8_t kind;              /* MV_RECT_*                                                               */
    uint8_t rest_rgb[3];       /* gauges: colour of the unfilled part                                     */
    uint8_t value_index;       /* gauges: which of the observation's values sets the filled length        */
} mv_rect;

/* Paint the primitives into an already rendered colour tensor, in place, after the render on `stream`, in list
 * order: a later primitive covers an earlier one.
 *   rgb    : device [N*A, H, W, 3] uint8.
 *   rects  : HOST memory, num_rects (1..MV_MAX_OVERLAY_RECTS) primitives, read before the call returns.
 *   values : [N*A, values_per_obs] float32 (0..MV_MAX_OVERLAY_VALUES per observation), host memory if
 *            src_is_device == 0 (validated: non-finite -> MV_ERR_ARG; copied on `stream`, which is waited for),
 *            else device memory; may be NULL when no primitive is a gauge.
 * A gauge of extent e (its width or height) shows n = floor(v*e + 0.5) filled columns or rows, clamped to 0..e,
 * computed in float32 (the indicator bar's rule; mv_draw_bars is one rightward gauge).  Depth is not touched.
 * Inactive environments (mv_set_active) are skipped.  With device values the call copies nothing to the host,
 * allocates nothing and waits for nothing, so it can be captured in a HIP graph.
 * Errors: MV_ERR_ARG (null, a primitive outside the image, unknown kind, value_index >= values_per_obs, too many
 * primitives or values), MV_ERR_HIP. */
int mv_draw_overlay(mv_batch* batch, uint8_t* rgb, const mv_rect* rects, int32_t num_rects, const float* values,
                    int32_t values_per_obs, int32_t src_is_device, void* hip_stream);

/* One simulator step for the whole batch in a single call (paper App. A.1: a vectorised interface, one
 * step for all N x M agents, with environments that reset on their own; Sec. 3.2: the state changes a
 * little per step and the cameras move with the agents).  In stream order the call applies this step's
 * voxel edits (mv_update_voxels), moves the cameras (mv_set_cameras), marks the environments whose
 * episode ended with this step as inactive (mv_set_active with the flags inverted), renders every other
 * environment (mv_render_batch without the aux outputs) and, if asked, paints the indicator bar
 * (mv_draw_bars) and then the overlay primitives (mv_draw_overlay).  Every pointer in mv_step_inputs is DEVICE memory on the batch's device and is not
 * validated; nothing is copied to the host, allocated or waited for, so the call can be captured in a
 * HIP graph.  The caller resets a finished environment by uploading its next world (mv_upload_worlds with
 * first_env, count) before the step in which it is no longer flagged.  The inactive set stays in force for
 * later mv_render_batch / mv_draw_bars calls until mv_set_active or the next mv_step replaces it.  The edit list
 * follows the rule of mv_update_voxels (all clears before all fills, one fill per voxel); a captured step keeps
 * all grid layers on chip (see mv_render_batch). */
typedef struct {
    int32_t        num_edits;      /* voxel edits of this step, >= 0                                   */
    const int32_t* edit_env;       /* [num_edits] environment of each edit; may be NULL if num_edits == 0 */
    const int32_t* edit_voxel;     /* [num_edits] linear voxel index                                   */
    const uint8_t* edit_material;  /* [num_edits] new material id, 0 = empty                           */
    const float*   cams;           /* [N*A, 5] (x, y, z, yaw, pitch), required                         */
    const int32_t* self_voxel;     /* [N*A] own-body voxel or -1; NULL = none                          */
    const uint8_t* done;           /* [N] non-zero = episode ended, do not render; NULL = render all   */
    const float*   bar_fraction;   /* [N*A] filled share of the bar; NULL = no bar                     */
    const mv_bar*  bar;            /* HOST pointer, read during the call; required if bar_fraction     */
    const mv_rect* overlay;        /* HOST pointer to num_overlay primitives, painted after the bar     */
    int32_t        num_overlay;    /* 0 = no overlay                                                    */
    int32_t        overlay_values_per_obs;  /* 0..MV_MAX_OVERLAY_VALUES                                 */
    const float*   overlay_values; /* [N*A, overlay_values_per_obs] gauge values; NULL if no gauge      */
} mv_step_inputs;

/* rgb, depth: as for mv_render_batch (device, caller-owned; frames of finished environments keep what
 * the tensors held).  Errors: those of the calls it is made of (MV_ERR_ARG for a null or negative
 * field, MV_ERR_STATE before every environment has a grid, MV_ERR_HIP); edits already enqueued when a
 * later part fails are not undone. */
int mv_step(mv_batch* batch, const mv_step_inputs* in, uint8_t* rgb, float* depth, void* hip_stream);

/* Pinned (page-locked) host memory for CPU consumers of the observations (paper Sec. 3.2: the images can
 * stay on the GPU for a GPU learner; a CPU learner or a logger reads them back).  Copies into memory
 * from mv_host_alloc run asynchronously at full PCIe rate; plain malloc'd memory also works with
 * mv_fetch_observations but makes that call wait for the copy.  mv_host_free(NULL) is a no-op; free
 * only after every copy into the block has completed.  Errors: MV_ERR_ARG, MV_ERR_HIP. */
int mv_host_alloc(void** out, size_t bytes);
void mv_host_free(void* ptr);

/* Copy observations first_obs .. first_obs+count-1 from the rendered device tensors to host memory on
 * `stream`, after the render on the same stream:
 *   rgb_dev, depth_dev   : the tensors given to mv_render_batch (device [N*A,H,W,3] uint8, [N*A,H,W] float32).
 *   rgb_host, depth_host : destination of count*H*W*3 bytes / count*H*W floats; either may be NULL to skip it
 *                          (then its device tensor may be NULL too).
 * Returns without synchronising: the host data is complete once the stream has passed this call
 * (hipStreamSynchronize or an event).  Errors: MV_ERR_ARG, MV_ERR_RANGE (observation range), MV_ERR_HIP. */
int mv_fetch_observations(mv_batch* batch, const uint8_t* rgb_dev, const float* depth_dev, int32_t first_obs,
                          int32_t count, uint8_t* rgb_host, float* depth_host, void* hip_stream);

/* The whole path in one call for callers that cannot allocate device memory: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Equivalent to mv_create_batch(cfg) + mv_upload_worlds +
 * mv_set_cameras + mv_render_batch (no aux outputs) on device inputs, but without a batch object: the working
 * memory a batch would own (occupancy bit rows, top layers, colour tables, camera records, pixel scalars) is a
 * fixed array of MV_NOALLOC_SCRATCH_BYTES inside the library's device image, one copy per GPU, held until the
 * process ends.  The call allocates nothing (no hipMalloc, hipFree or host heap), copies nothing to the host
 * and does not wait.
 *   voxels     : device [N, Z, Y, X] uint8 material ids; read by the kernels of this call, not copied: keep it
 *                unchanged until the stream has passed the call.  Not validated (ids above num_materials are
 *                clamped when shading).
 *   palette    : device [N, num_materials+1, 3] uint8, required.
 *   cams       : device [N*A, 5] float32 (x, y, z, yaw, pitch); self_voxel : device [N*A] int32 or NULL.
 *   rgb, depth : device outputs as for mv_render_batch.
 * Working memory needed: N * (8 * (Z*Y*ceil(X/64) + Z*X*ceil(Y/64)) + 28 * (num_materials+1) + 4) + 64 * N*A +
 * 4 * (W + H) bytes plus up to 256 bytes of padding per piece; a configuration that needs more than
 * MV_NOALLOC_SCRATCH_BYTES is refused with MV_ERR_CAPACITY before anything is enqueued (256 environments x 4
 * agents of 40x40x16 voxels need 2.8 MB).  Every call on a GPU uses that GPU's one array: calls that overlap
 * on one GPU (two streams, two threads) race; order them.  Each call rewrites every word it later reads, so
 * what an earlier call left behind never shows.  cfg->tiles_per_block is honoured as in mv_create_batch.
 * Errors: MV_ERR_ARG, MV_ERR_CAPACITY, MV_ERR_HIP. */
#define MV_NOALLOC_SCRATCH_BYTES (8u << 20)
int mv_render_worlds_noalloc(const mv_config* cfg, const uint8_t* voxels, const uint8_t* palette,
                             const float* cams, const int32_t* self_voxel, uint8_t* rgb, float* depth,
                             void* hip_stream);

/* Free the batch and its device memory (synchronises the device first).  NULL is a no-op. */
void mv_destroy(mv_batch* batch);

/* Description of the last error on this thread ("" if none).  Never NULL. */
const char* mv_last_error(void);

/* Introspection for tests and benchmarks (device pointers stay owned by the batch):
 *   mv_debug_occupancy : device pointers to the packed occupancy "bit rows" of environment `env`.
 *                        x rows: Z*Y rows of *x_row_words 64-bit words, row k*Y+j, bit i of the row
 *                        is voxel (i,j,k); y rows: Z*X rows of *y_row_words words, row k*X+i, bit j
 *                        is voxel (i,j,k); *top_layer points to one int32: 1 + the highest layer k
 *                        that holds a solid voxel (0 for an empty grid).
 *   mv_debug_camera_records : device pointer to the [N*A] 64-byte camera records
 *                        (float P[3], F[3], R[3], U[3]; int32 self_lo, self_hi; 8 bytes pad).
 *   mv_debug_set_staged_layers : the render kernel keeps only the lowest layers of a grid on chip, as many
 *                        as the tallest world uploaded so far needs (it learns that number from its own
 *                        kernels, without synchronising); an environment that needs more is traced
 *                        through device memory instead, with identical results.  This call fixes the number
 *                        (1..Z) so that tests can reach that path; 0 returns to the automatic choice.
 *                        Errors: MV_ERR_ARG, MV_ERR_RANGE.
 *   mv_debug_launch_shape : how a render of this configuration with `staged_layers` layers on chip (0 = all Z)
 *                        is laid out, computed on the host without touching a GPU: *shape receives the LDS bytes and
 *                        threads of a workgroup and the work list (workgroup b of the launch belongs to XCD b mod 8
 *                        and is number s = b div 8 there; an XCD renders the observations x*obs_per_xcd ..
 *                        (x+1)*obs_per_xcd-1 that exist; s < obs_body_per_xcd*blocks_per_obs: observation
 *                        s div blocks_per_obs of the range, strip s mod blocks_per_obs of tiles_per_block tiles;
 *                        later workgroups cut the remaining observations into blocks_per_obs_tail strips of
 *                        tiles_per_block_tail tiles; a strip is tiles strip*t .. min((strip+1)*t, tiles_per_obs)-1
 *                        of the observation's tiles_x-wide, row-major grid of 8x8-pixel tiles; where an observation has
 *                        an even number of strips, which workgroup takes which of them is rotated by a hash of the
 *                        observation index).
 *                        Errors: those of mv_create_batch for the configuration. */
int mv_debug_occupancy(mv_batch* batch, int32_t env, const uint64_t** x_rows, int32_t* x_row_words,
                       const uint64_t** y_rows, int32_t* y_row_words, const int32_t** top_layer);
int mv_debug_camera_records(mv_batch* batch, const void** records);
int mv_debug_set_staged_layers(mv_batch* batch, int32_t layers);
typedef struct {
    int32_t lds_bytes, threads;
    int32_t tiles_x, tiles_per_obs;
    int32_t tiles_per_block, blocks_per_obs, tiles_per_block_tail, blocks_per_obs_tail;
    int32_t num_obs, obs_per_xcd, obs_body_per_xcd;
    uint32_t blocks_per_xcd;       /* the launch has 8 * blocks_per_xcd workgroups */
} mv_launch_shape;
int mv_debug_launch_shape(const mv_config* cfg, int32_t staged_layers, mv_launch_shape* shape);

#ifdef __cplusplus
}
#endif
#endif
