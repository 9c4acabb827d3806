/*
 * Algorithm O of the CPU oracle: float64 3D-DDA ray casting of batched voxel worlds.
 * TEST INFRASTRUCTURE ONLY -- see mv_oracle.h.  Nothing here is shared with the HIP library.
 *
 * Per observation o = env*A + agent (paper App. A.1: a vector of N x M observations), per pixel
 * row r (0 = top) and column c (0 = left):
 *   1. camera basis in float64 from (yaw, pitch), scaled by tan(hfov/2) and the aspect ratio,
 *      then rounded to twelve float32 numbers: the camera IS those twelve numbers;
 *   2. pixel-centre scalars sx = (2c+1-W)/W, sy = (H-2r-1)/H in float32;
 *   3. ray direction d = F + sx*R + sy*U with two float32 fused multiply-adds per axis (not
 *      normalised, so the ray parameter t is planar depth along the forward axis);
 *   4. everything after that in float64: clip against the grid box, walk voxel to voxel
 *      picking the nearest of the three next plane crossings (ties: x before y before z), stop
 *      at the first solid voxel that is not the camera's own body;
 *   5. colour = palette[material] * intensity[face], rounded in float32; depth = (float)t.
 */
#include "mv_oracle.h"

#include <math.h>
#include <pthread.h>
#include <stdlib.h>
#include <string.h>

struct mvo_batch {
    mvo_config cfg;
    double   tan_half_x, tan_half_y;
    float    intensity[7];
    uint8_t* vox;        /* [N][Z][Y][X] */
    uint8_t* pal;        /* [N][M+1][3]  */
    uint8_t* env_ready;  /* [N] grid uploaded; */
    uint8_t* pal_ready;  /* [N] palette uploaded */
    float*   rec;        /* [N*A][12] P,F,R,U */
    int32_t* self_voxel; /* [N*A] */
    int      cams_ready;
};

typedef struct {
    uint8_t rgb[3];
    float   depth;
    uint8_t material;
    int32_t hit_index;
    uint8_t face;
    int32_t steps;
    double  edge_margin;
    double  t;
} pixel_result;

static size_t voxels_per_env(const mvo_batch* b)
{
    return (size_t)b->cfg.grid_x * (size_t)b->cfg.grid_y * (size_t)b->cfg.grid_z;
}

int mvo_create(const mvo_config* cfg, mvo_batch** out)
{
    if (!cfg || !out) return -1;
    if (cfg->num_envs <= 0 || cfg->agents_per_env <= 0 || cfg->grid_x <= 0 || cfg->grid_y <= 0 ||
        cfg->grid_z <= 0 || cfg->width <= 0 || cfg->height <= 0 || cfg->num_materials < 1 ||
        cfg->num_materials > 255)
        return -1;
    if (!(cfg->hfov_rad > 0.0f) || !(cfg->hfov_rad < 3.14159f)) return -1;
    double lx = cfg->light_dir[0], ly = cfg->light_dir[1], lz = cfg->light_dir[2];
    double ln = sqrt(lx * lx + ly * ly + lz * lz);
    if (!(ln > 0.0) || !isfinite(ln)) return -1;

    mvo_batch* b = (mvo_batch*)calloc(1, sizeof(*b));
    if (!b) return -1;
    b->cfg = *cfg;
    b->tan_half_x = tan(0.5 * (double)cfg->hfov_rad);
    b->tan_half_y = b->tan_half_x * (double)cfg->height / (double)cfg->width;   /* square pixels */

    /* Lambert term of the six axis-aligned outward normals against the unit light direction:
     * face 0:-x 1:+x 2:-y 3:+y 4:-z 5:+z, 6 = origin inside a solid (ambient only). */
    const double L[3] = { lx / ln, ly / ln, lz / ln };
    for (int f = 0; f < 6; ++f) {
        double ndotl = (f & 1) ? L[f >> 1] : -L[f >> 1];
        if (ndotl < 0.0) ndotl = 0.0;
        b->intensity[f] = (float)((double)cfg->ambient + (double)cfg->diffuse * ndotl);
    }
    b->intensity[6] = (float)(double)cfg->ambient;

    size_t N = (size_t)cfg->num_envs, NA = N * (size_t)cfg->agents_per_env;
    b->vox = (uint8_t*)calloc(N * voxels_per_env(b), 1);
    b->pal = (uint8_t*)calloc(N * (size_t)(cfg->num_materials + 1) * 3, 1);
    b->env_ready = (uint8_t*)calloc(N, 1);
    b->pal_ready = (uint8_t*)calloc(N, 1);
    b->rec = (float*)calloc(NA * 12, sizeof(float));
    b->self_voxel = (int32_t*)malloc(NA * sizeof(int32_t));
    if (!b->vox || !b->pal || !b->env_ready || !b->pal_ready || !b->rec || !b->self_voxel) {
        mvo_destroy(b);
        return -1;
    }
    for (size_t i = 0; i < NA; ++i) b->self_voxel[i] = -1;
    *out = b;
    return 0;
}

void mvo_destroy(mvo_batch* b)
{
    if (!b) return;
    free(b->vox); free(b->pal); free(b->env_ready); free(b->pal_ready);
    free(b->rec); free(b->self_voxel);
    free(b);
}

int mvo_upload_worlds(mvo_batch* b, int32_t first_env, int32_t count, const uint8_t* voxels,
                      const uint8_t* palette)
{
    if (!b || !voxels) return -1;
    if (first_env < 0 || count <= 0 || first_env > b->cfg.num_envs - count) return -3;
    size_t per = voxels_per_env(b);
    for (size_t i = 0; i < (size_t)count * per; ++i)
        if (voxels[i] > b->cfg.num_materials) return -3;
    memcpy(b->vox + (size_t)first_env * per, voxels, (size_t)count * per);
    memset(b->env_ready + first_env, 1, (size_t)count);
    if (palette) {
        size_t pp = (size_t)(b->cfg.num_materials + 1) * 3;
        memcpy(b->pal + (size_t)first_env * pp, palette, (size_t)count * pp);
        memset(b->pal_ready + first_env, 1, (size_t)count);
    }
    return 0;
}

int mvo_update_voxels(mvo_batch* b, int32_t count, const int32_t* env, const int32_t* voxel_index,
                      const uint8_t* material)
{
    if (!b || count < 0) return -1;
    if (count == 0) return 0;
    if (!env || !voxel_index || !material) return -1;
    size_t per = voxels_per_env(b);
    for (int32_t e = 0; e < count; ++e) {
        if (env[e] < 0 || env[e] >= b->cfg.num_envs) return -3;
        if (voxel_index[e] < 0 || (size_t)voxel_index[e] >= per) return -3;
        if (material[e] > b->cfg.num_materials) return -3;
        if (!b->env_ready[env[e]]) return -2;
    }
    for (int32_t e = 0; e < count; ++e)
        b->vox[(size_t)env[e] * per + (size_t)voxel_index[e]] = material[e];
    return 0;
}

int mvo_set_cameras(mvo_batch* b, const float* cams, const int32_t* self_voxel)
{
    if (!b || !cams) return -1;
    size_t NA = (size_t)b->cfg.num_envs * (size_t)b->cfg.agents_per_env;
    for (size_t i = 0; i < NA * 5; ++i)
        if (!isfinite(cams[i])) return -1;
    for (size_t o = 0; o < NA; ++o) {
        const float* c = cams + 5 * o;
        double yaw = (double)c[3], pitch = (double)c[4];
        double cy = cos(yaw), sy = sin(yaw), cp = cos(pitch), sp = sin(pitch);
        double fwd[3]   = { cp * cy, cp * sy, sp };
        double right[3] = { sy, -cy, 0.0 };
        double up[3]    = { -sp * cy, -sp * sy, cp };
        float* r = b->rec + 12 * o;
        for (int a = 0; a < 3; ++a) {
            r[a]     = c[a];
            r[3 + a] = (float)fwd[a];
            r[6 + a] = (float)(b->tan_half_x * right[a]);
            r[9 + a] = (float)(b->tan_half_y * up[a]);
        }
        b->self_voxel[o] = self_voxel ? self_voxel[o] : -1;
    }
    b->cams_ready = 1;
    return 0;
}

int mvo_draw_bars(const mvo_batch* b, int32_t first_obs, int32_t count, uint8_t* rgb, const float* fraction,
                  int32_t x, int32_t y, int32_t width, int32_t height, const uint8_t fill_rgb[3],
                  const uint8_t empty_rgb[3], const uint8_t* active)
{
    if (!b || !rgb || !fraction || !fill_rgb || !empty_rgb) return -1;
    const int32_t W = b->cfg.width, H = b->cfg.height;
    if (width <= 0 || height <= 0 || x < 0 || y < 0 || x > W - width || y > H - height) return -1;
    if (first_obs < 0 || count <= 0 || first_obs > b->cfg.num_envs * b->cfg.agents_per_env - count) return -3;
    for (int32_t o = 0; o < count; ++o) {
        if (active && !active[(first_obs + o) / b->cfg.agents_per_env]) continue;
        volatile float prod = fraction[o] * (float)width;
        volatile float sum = prod + 0.5f;
        float cols = floorf(sum);
        if (!(cols > 0.0f)) cols = 0.0f;
        if (cols > (float)width) cols = (float)width;
        const int32_t filled = (int32_t)cols;
        for (int32_t r = 0; r < height; ++r)
            for (int32_t c = 0; c < width; ++c) {
                uint8_t* px = rgb + (((size_t)o * H + (size_t)(y + r)) * W + (size_t)(x + c)) * 3;
                const uint8_t* col = c < filled ? fill_rgb : empty_rgb;
                px[0] = col[0]; px[1] = col[1]; px[2] = col[2];
            }
    }
    return 0;
}

int mvo_draw_overlay(const mvo_batch* b, int32_t first_obs, int32_t count, uint8_t* rgb, const mvo_rect* rects,
                     int32_t num_rects, const float* values, int32_t values_per_obs, const uint8_t* active)
{
    if (!b || !rgb || !rects || num_rects <= 0 || values_per_obs < 0) return -1;
    const int32_t W = b->cfg.width, H = b->cfg.height;
    if (first_obs < 0 || count <= 0 || first_obs > b->cfg.num_envs * b->cfg.agents_per_env - count) return -3;
    for (int32_t k = 0; k < num_rects; ++k) {
        const mvo_rect* q = &rects[k];
        if (q->width <= 0 || q->height <= 0 || q->x < 0 || q->y < 0 || q->x > W - q->width || q->y > H - q->height)
            return -1;
        if (q->kind > 2) return -1;
        if (q->kind != 0 && (!values || q->value_index >= values_per_obs)) return -1;
    }
    for (int32_t o = 0; o < count; ++o) {
        if (active && !active[(first_obs + o) / b->cfg.agents_per_env]) continue;
        uint8_t* img = rgb + (size_t)o * H * W * 3;
        for (int32_t k = 0; k < num_rects; ++k) {           /* in list order: later primitives paint over earlier ones */
            const mvo_rect* q = &rects[k];
            int32_t filled = 0;
            if (q->kind != 0) {
                const int32_t extent = q->kind == 1 ? q->width : q->height;
                volatile float prod = values[(size_t)o * values_per_obs + q->value_index] * (float)extent;
                volatile float sum = prod + 0.5f;
                float n = floorf(sum);
                if (!(n > 0.0f)) n = 0.0f;
                if (n > (float)extent) n = (float)extent;
                filled = (int32_t)n;
            }
            for (int32_t r = 0; r < q->height; ++r)
                for (int32_t c = 0; c < q->width; ++c) {
                    int in_front = 1;                                       /* kind 0: the whole rectangle */
                    if (q->kind == 1) in_front = c < filled;                /* columns from the left edge */
                    if (q->kind == 2) in_front = q->height - 1 - r < filled; /* rows from the bottom edge */
                    const uint8_t* col = in_front ? q->rgb : q->rest_rgb;
                    uint8_t* px = img + ((size_t)(q->y + r) * W + (size_t)(q->x + c)) * 3;
                    px[0] = col[0]; px[1] = col[1]; px[2] = col[2];
                }
        }
    }
    return 0;
}

int mvo_camera_record(const mvo_batch* b, int32_t obs, float rec[12])
{
    if (!b || !rec || !b->cams_ready) return -1;
    if (obs < 0 || obs >= b->cfg.num_envs * b->cfg.agents_per_env) return -3;
    memcpy(rec, b->rec + 12 * (size_t)obs, 12 * sizeof(float));
    return 0;
}

static void pixel_ray(const mvo_batch* b, int32_t obs, int32_t row, int32_t col, float dir[3])
{
    const int32_t W = b->cfg.width, H = b->cfg.height;
    const float* rec = b->rec + 12 * (size_t)obs;
    float sx = (float)(2 * col + 1 - W) / (float)W;
    float sy = (float)(H - 2 * row - 1) / (float)H;
    for (int a = 0; a < 3; ++a)
        dir[a] = fmaf(sy, rec[9 + a], fmaf(sx, rec[6 + a], rec[3 + a]));
}

int mvo_pixel_ray(const mvo_batch* b, int32_t obs, int32_t row, int32_t col, float dir[3])
{
    if (!b || !dir || !b->cams_ready) return -1;
    if (obs < 0 || obs >= b->cfg.num_envs * b->cfg.agents_per_env || row < 0 ||
        row >= b->cfg.height || col < 0 || col >= b->cfg.width)
        return -3;
    pixel_ray(b, obs, row, col, dir);
    return 0;
}

int mvo_face_intensity(const mvo_batch* b, float out[7])
{
    if (!b || !out) return -1;
    memcpy(out, b->intensity, sizeof(b->intensity));
    return 0;
}

uint8_t mvo_quantise(uint8_t palette_value, float intensity)
{
    volatile float prod = (float)palette_value * intensity;   /* one float32 rounding */
    volatile float sum = prod + 0.5f;                          /* a second one        */
    float q = floorf(sum);
    if (q > 255.0f) q = 255.0f;
    if (q < 0.0f) q = 0.0f;
    return (uint8_t)q;
}

/* In-plane distance of a crossing point to the nearest grid line of the two other axes. */
static double crossing_margin(const double P[3], const double d[3], double t, int axis)
{
    double m = INFINITY;
    for (int a = 0; a < 3; ++a) {
        if (a == axis) continue;
        double q = P[a] + t * d[a];
        double dist = fabs(q - nearbyint(q));
        if (dist < m) m = dist;
    }
    return m;
}

static void trace_pixel(const mvo_batch* b, int32_t obs, int32_t row, int32_t col,
                        pixel_result* out)
{
    const int32_t dim[3] = { b->cfg.grid_x, b->cfg.grid_y, b->cfg.grid_z };
    const int32_t env = obs / b->cfg.agents_per_env;
    const uint8_t* vox = b->vox + (size_t)env * voxels_per_env(b);
    const uint8_t* pal = b->pal + (size_t)env * (size_t)(b->cfg.num_materials + 1) * 3;
    const int32_t self_lo = b->self_voxel[obs];
    const int32_t self_hi = self_lo >= 0 ? self_lo + dim[0] * dim[1] : -1;

    float dirf[3];
    pixel_ray(b, obs, row, col, dirf);
    const float* rec = b->rec + 12 * (size_t)obs;
    const double P[3] = { (double)rec[0], (double)rec[1], (double)rec[2] };
    const double d[3] = { (double)dirf[0], (double)dirf[1], (double)dirf[2] };

    out->rgb[0] = b->cfg.sky_rgb[0]; out->rgb[1] = b->cfg.sky_rgb[1]; out->rgb[2] = b->cfg.sky_rgb[2];
    out->depth = 0.0f; out->material = 0; out->hit_index = -1; out->face = MVO_FACE_MISS;
    out->steps = 0; out->edge_margin = INFINITY; out->t = 0.0;

    /* grid entry */
    double t0 = 0.0;
    int entry_axis = -1;
    int inside = 1;
    for (int a = 0; a < 3; ++a)
        if (P[a] < 0.0 || P[a] > (double)dim[a]) inside = 0;
    if (!inside) {
        double t_near = -INFINITY, t_far = INFINITY;
        for (int a = 0; a < 3; ++a) {
            if (d[a] == 0.0) {
                if (P[a] < 0.0 || P[a] > (double)dim[a]) return;        /* parallel, outside */
                continue;
            }
            double ta = ((d[a] > 0.0 ? 0.0 : (double)dim[a]) - P[a]) / d[a];
            double tb = ((d[a] > 0.0 ? (double)dim[a] : 0.0) - P[a]) / d[a];
            if (ta > t_near) { t_near = ta; entry_axis = a; }
            if (tb < t_far) t_far = tb;
        }
        if (t_near > t_far || t_far < 0.0) {
            /* The ray passes the whole grid by.  If it does so within a hair of the rim of the boundary face it
               would have entered through, that is a tie like any grazed voxel edge (enter the voxel at the rim,
               or miss everything): the margin is how far outside that face's rectangle the ray meets the face's
               plane, the larger of its excesses along the two other axes. */
            if (t_near > 0.0 && t_far >= 0.0 && entry_axis >= 0) {
                double worst = 0.0;
                for (int a = 0; a < 3; ++a) {
                    if (a == entry_axis) continue;
                    double q = P[a] + t_near * d[a];
                    double excess = q < 0.0 ? -q : (q > (double)dim[a] ? q - (double)dim[a] : 0.0);
                    if (excess > worst) worst = excess;
                }
                out->edge_margin = worst;
            }
            return;
        }
        if (t_near > 0.0) t0 = t_near; else entry_axis = -1;
    }

    int32_t cell[3];
    for (int a = 0; a < 3; ++a) {
        double q = floor(P[a] + t0 * d[a]);
        if (q < 0.0) q = 0.0;
        if (q > (double)(dim[a] - 1)) q = (double)(dim[a] - 1);
        cell[a] = (int32_t)q;
    }
    if (entry_axis >= 0) {
        cell[entry_axis] = d[entry_axis] > 0.0 ? 0 : dim[entry_axis] - 1;
        out->edge_margin = crossing_margin(P, d, t0, entry_axis);
    }

    int32_t step[3];
    double t_max[3];
    for (int a = 0; a < 3; ++a) {
        if (d[a] > 0.0)      { step[a] = 1;  t_max[a] = ((double)(cell[a] + 1) - P[a]) / d[a]; }
        else if (d[a] < 0.0) { step[a] = -1; t_max[a] = ((double)cell[a] - P[a]) / d[a]; }
        else                 { step[a] = 0;  t_max[a] = INFINITY; }
    }

    double t_hit = t0;
    int face = entry_axis >= 0 ? 2 * entry_axis + (d[entry_axis] < 0.0 ? 1 : 0) : MVO_FACE_INSIDE;
    int32_t idx = (cell[2] * dim[1] + cell[1]) * dim[0] + cell[0];
    int found = vox[idx] != 0 && idx != self_lo && idx != self_hi;

    const int32_t max_steps = dim[0] + dim[1] + dim[2] + 3;
    while (!found && out->steps < max_steps) {
        int axis;
        if (t_max[0] <= t_max[1] && t_max[0] <= t_max[2]) axis = 0;
        else if (t_max[1] <= t_max[2]) axis = 1;
        else axis = 2;
        if (t_max[axis] == INFINITY) return;        /* direction is the zero vector */
        t_hit = t_max[axis];
        cell[axis] += step[axis];
        out->steps += 1;
        /* every plane crossing counts for the margin, the one through the grid boundary included: a ray
           that leaves within a hair of the line where the boundary meets a voxel face is as much a tie
           (leave, or enter that voxel) as one that grazes an edge inside the grid */
        double m = crossing_margin(P, d, t_hit, axis);
        if (m < out->edge_margin) out->edge_margin = m;
        if (cell[axis] < 0 || cell[axis] >= dim[axis]) return;          /* left the grid: miss */
        double next_plane = (double)(cell[axis] + (step[axis] > 0 ? 1 : 0));
        t_max[axis] = (next_plane - P[axis]) / d[axis];
        face = 2 * axis + (step[axis] < 0 ? 1 : 0);
        idx = (cell[2] * dim[1] + cell[1]) * dim[0] + cell[0];
        found = vox[idx] != 0 && idx != self_lo && idx != self_hi;
    }
    if (!found) return;

    out->t = t_hit;
    out->depth = (float)t_hit;
    out->hit_index = idx;
    out->material = vox[idx];
    out->face = (uint8_t)face;
    const float I = b->intensity[face];
    for (int ch = 0; ch < 3; ++ch)
        out->rgb[ch] = mvo_quantise(pal[3 * (size_t)out->material + ch], I);
}

typedef struct {
    const mvo_batch* b;
    int32_t first_obs, count, tid, nthreads;
    uint8_t* rgb; float* depth; uint8_t* material; int32_t* hit_index; uint8_t* face;
    int32_t* steps; double* edge_margin; double* t_exact;
} render_job;

static void store_pixel(const pixel_result* p, size_t i, uint8_t* rgb, float* depth,
                        uint8_t* material, int32_t* hit_index, uint8_t* face, int32_t* steps,
                        double* edge_margin, double* t_exact)
{
    if (rgb) { rgb[3 * i] = p->rgb[0]; rgb[3 * i + 1] = p->rgb[1]; rgb[3 * i + 2] = p->rgb[2]; }
    if (depth) depth[i] = p->depth;
    if (material) material[i] = p->material;
    if (hit_index) hit_index[i] = p->hit_index;
    if (face) face[i] = p->face;
    if (steps) steps[i] = p->steps;
    if (edge_margin) edge_margin[i] = p->edge_margin;
    if (t_exact) t_exact[i] = p->t;
}

static void* render_worker(void* arg)
{
    render_job* j = (render_job*)arg;
    const int32_t W = j->b->cfg.width, H = j->b->cfg.height;
    for (int32_t k = j->tid; k < j->count; k += j->nthreads) {
        for (int32_t r = 0; r < H; ++r)
            for (int32_t c = 0; c < W; ++c) {
                pixel_result p;
                trace_pixel(j->b, j->first_obs + k, r, c, &p);
                size_t i = ((size_t)k * (size_t)H + (size_t)r) * (size_t)W + (size_t)c;
                store_pixel(&p, i, j->rgb, j->depth, j->material, j->hit_index, j->face,
                            j->steps, j->edge_margin, j->t_exact);
            }
    }
    return NULL;
}

static int check_ready(const mvo_batch* b, int32_t obs)
{
    int32_t env = obs / b->cfg.agents_per_env;
    return b->cams_ready && b->env_ready[env] && b->pal_ready[env];
}

int mvo_render(mvo_batch* b, int32_t first_obs, int32_t count, uint8_t* rgb, float* depth,
               uint8_t* material, int32_t* hit_index, uint8_t* face, int32_t* steps,
               double* edge_margin, double* t_exact, int32_t num_threads)
{
    if (!b) return -1;
    int32_t NA = b->cfg.num_envs * b->cfg.agents_per_env;
    if (first_obs < 0 || count <= 0 || first_obs > NA - count) return -3;
    for (int32_t o = first_obs; o < first_obs + count; ++o)
        if (!check_ready(b, o)) return -2;
    if (num_threads < 1) num_threads = 1;
    if (num_threads > count) num_threads = count;
    if (num_threads > 256) num_threads = 256;

    render_job jobs[256];
    pthread_t threads[256];
    for (int32_t t = 0; t < num_threads; ++t) {
        render_job j = { b, first_obs, count, t, num_threads, rgb, depth, material, hit_index,
                         face, steps, edge_margin, t_exact };
        jobs[t] = j;
    }
    if (num_threads == 1) { render_worker(&jobs[0]); return 0; }
    int started = 0;
    for (; started < num_threads; ++started)
        if (pthread_create(&threads[started], NULL, render_worker, &jobs[started]) != 0) break;
    for (int32_t t = started; t < num_threads; ++t) render_worker(&jobs[t]);  /* fallback: inline */
    for (int32_t t = 0; t < started; ++t) pthread_join(threads[t], NULL);
    return 0;
}

int mvo_render_pixels(mvo_batch* b, int64_t n, const int32_t* obs, const int32_t* row,
                      const int32_t* col, uint8_t* rgb, float* depth, uint8_t* material,
                      int32_t* hit_index, uint8_t* face, int32_t* steps, double* edge_margin,
                      double* t_exact)
{
    if (!b || !obs || !row || !col || n < 0) return -1;
    int32_t NA = b->cfg.num_envs * b->cfg.agents_per_env;
    for (int64_t i = 0; i < n; ++i) {
        if (obs[i] < 0 || obs[i] >= NA || row[i] < 0 || row[i] >= b->cfg.height || col[i] < 0 ||
            col[i] >= b->cfg.width)
            return -3;
        if (!check_ready(b, obs[i])) return -2;
    }
    for (int64_t i = 0; i < n; ++i) {
        pixel_result p;
        trace_pixel(b, obs[i], row[i], col[i], &p);
        store_pixel(&p, (size_t)i, rgb, depth, material, hit_index, face, steps, edge_margin,
                    t_exact);
    }
    return 0;
}
