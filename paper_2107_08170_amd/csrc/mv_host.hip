// Host runtime of the batched voxel-world renderer: the batch object, argument checking, device
// memory, and the C ABI declared in include/mv.h.  Every arithmetic step of the render path runs
// in the kernels of mv_kernels.hip; this file only validates, allocates, copies and launches.
#include "mv.h"
#include "mv_internal.h"

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

namespace {

thread_local char g_error[512] = "";

int fail(int code, const char* fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_error, sizeof(g_error), fmt, ap);
    va_end(ap);
    return code;
}

#define MV_HIP(expr)                                                                                  \
    do {                                                                                              \
        hipError_t e_ = (expr);                                                                       \
        if (e_ != hipSuccess)                                                                         \
            return fail(MV_ERR_HIP, "%s failed: %s (%s:%d)", #expr, hipGetErrorString(e_), __FILE__, __LINE__); \
    } while (0)

// Makes the batch's device current for the duration of a call and restores the caller's.
class DeviceScope {
public:
    explicit DeviceScope(int device) : ok_(false), prev_(-1)
    {
        if (hipGetDevice(&prev_) != hipSuccess) return;
        if (prev_ != device && hipSetDevice(device) != hipSuccess) return;
        ok_ = true;
        target_ = device;
    }
    ~DeviceScope()
    {
        if (ok_ && prev_ != target_) (void)hipSetDevice(prev_);
    }
    bool ok() const { return ok_; }

private:
    bool ok_;
    int prev_, target_ = -1;
};

}  // namespace

struct mv_batch {
    mv_config cfg{};
    int num_obs = 0;
    int voxels_per_env = 0;
    mv::GridLayout layout{};
    mv::LdsPlan plan{};
    int materials_plus_one = 0;
    double tan_half_x = 0, tan_half_y = 0;
    float intensity[mv::kNumFaces] = {};

    uint8_t* d_vox = nullptr;
    const uint8_t* borrowed_vox = nullptr;   // the caller's material array while the batch borrows it, else null
    uint64_t* d_bits = nullptr;
    int32_t* d_ztop = nullptr;
    uint8_t* d_palette = nullptr;
    uint32_t* d_lut = nullptr;
    float* d_sx = nullptr;
    float* d_sy = nullptr;
    uint8_t* d_active = nullptr;      // [N] render mask
    bool all_active = true;
    float* d_fraction = nullptr;      // [N*A] staging for host-supplied bar fractions
    float* d_overlay_values = nullptr; // [N*A][MV_MAX_OVERLAY_VALUES] staging for host-supplied gauge values
    uint8_t* d_edits = nullptr;       // staging for host-supplied voxel edits and moves, 13 bytes per entry (grown on demand)
    size_t edits_capacity = 0;        // in edits
    float* d_cams = nullptr;          // staging for host-supplied cameras
    int32_t* d_self = nullptr;
    mv::CameraRecord* d_rec = nullptr;
    // tallest world so far: exact on the device, and a pinned host word that kernels keep up to date and
    // that mv_render_batch reads without synchronising to choose how many layers to stage
    int32_t* d_height = nullptr;
    int32_t* h_height = nullptr;          // pinned host memory
    int32_t* h_height_dev = nullptr;      // the same word as the device addresses it
    int forced_layers = 0;                // debug override (0 = automatic)

    std::vector<uint8_t> env_has_grid, env_has_palette;
    int envs_with_grid = 0, envs_with_palette = 0;
    bool cameras_set = false;
};

static void free_batch(mv_batch* b)
{
    if (!b) return;
    (void)hipFree(b->d_vox); (void)hipFree(b->d_bits); (void)hipFree(b->d_ztop); (void)hipFree(b->d_palette); (void)hipFree(b->d_lut);
    (void)hipFree(b->d_sx); (void)hipFree(b->d_sy); (void)hipFree(b->d_cams); (void)hipFree(b->d_self);
    (void)hipFree(b->d_rec); (void)hipFree(b->d_edits); (void)hipFree(b->d_active); (void)hipFree(b->d_fraction);
    (void)hipFree(b->d_overlay_values);
    (void)hipFree(b->d_height);
    if (b->h_height) (void)hipHostFree(b->h_height);
    delete b;
}

// Field checks shared by every call that takes a configuration; `who` prefixes the message.  On success
// *plan_out holds the LDS plan with all Z layers staged.
static int check_config(const mv_config* cfg, const char* who, mv::GridLayout* layout_out, mv::LdsPlan* plan_out)
{
    if (cfg->num_envs <= 0 || cfg->agents_per_env <= 0)
        return fail(MV_ERR_ARG, "%s: num_envs and agents_per_env must be positive", who);
    if (cfg->grid_x <= 0 || cfg->grid_y <= 0 || cfg->grid_z <= 0)
        return fail(MV_ERR_ARG, "%s: grid dimensions must be positive", who);
    if (cfg->width <= 0 || cfg->height <= 0 || cfg->width > 16384 || cfg->height > 16384)
        return fail(MV_ERR_ARG, "%s: image size must be in 1..16384", who);
    if (!(cfg->hfov_rad > 0.0f) || !(cfg->hfov_rad < 3.14159f))
        return fail(MV_ERR_ARG, "%s: hfov_rad must lie in (0, pi)", who);
    if (cfg->num_materials < 1 || cfg->num_materials > 255)
        return fail(MV_ERR_ARG, "%s: num_materials must be in 1..255", who);
    if (cfg->coarse_level > 1) return fail(MV_ERR_ARG, "%s: coarse_level must be 0 or 1", who);
    if (cfg->tiles_per_block < 0) return fail(MV_ERR_ARG, "%s: tiles_per_block must be >= 0", who);
    if (cfg->device < 0) return fail(MV_ERR_ARG, "%s: device must be >= 0", who);
    const double lx = cfg->light_dir[0], ly = cfg->light_dir[1], lz = cfg->light_dir[2];
    const double ln = std::sqrt(lx * lx + ly * ly + lz * lz);
    if (!(ln > 0.0) || !std::isfinite(ln)) return fail(MV_ERR_ARG, "%s: light_dir must be finite and non-zero", who);
    if (!std::isfinite(cfg->ambient) || !std::isfinite(cfg->diffuse))
        return fail(MV_ERR_ARG, "%s: ambient/diffuse must be finite", who);

    const long long voxels = (long long)cfg->grid_x * cfg->grid_y * cfg->grid_z;
    if (voxels > (1ll << 30)) return fail(MV_ERR_CAPACITY, "%s: grid too large", who);
    const long long num_obs = (long long)cfg->num_envs * cfg->agents_per_env;
    if (num_obs > (1ll << 24)) return fail(MV_ERR_ARG, "%s: more than 2^24 observations", who);
    const mv::GridLayout layout = mv::make_layout(cfg->grid_x, cfg->grid_y, cfg->grid_z);
    const mv::LdsPlan plan = mv::plan_lds(layout, cfg->width, cfg->height, cfg->num_materials + 1, cfg->grid_z,
                                          cfg->coarse_level != 0);
    if (plan.bytes == 0)
        return fail(MV_ERR_CAPACITY, "%s: the occupancy bit rows of one %dx%dx%d grid do not fit in %zu bytes of LDS", who,
                    cfg->grid_x, cfg->grid_y, cfg->grid_z, mv::kLdsBudget);

    // the pack kernel keeps one whole z layer per wave in LDS
    if (mv::pack_lds_bytes(layout) + mv::kPackStaticLds > mv::kLdsBudget)
        return fail(MV_ERR_CAPACITY, "%s: one %dx%d layer (x4 waves) does not fit in %zu bytes of LDS while packing", who,
                    cfg->grid_x, cfg->grid_y, mv::kLdsBudget);
    *layout_out = layout;
    *plan_out = plan;
    return MV_OK;
}

// Face intensities (flat Lambert shading): every face code has an outward unit normal, and a face is lit by
// ambient + diffuse * (how far its normal leans towards the light); faces turned away from the light, and
// the "inside" code, get the ambient term alone.
static void face_intensities(const mv_config& cfg, float out[mv::kNumFaces])
{
    static const signed char kNormal[6][3] = { { -1, 0, 0 }, { 1, 0, 0 }, { 0, -1, 0 }, { 0, 1, 0 }, { 0, 0, -1 }, { 0, 0, 1 } };
    const double lx = cfg.light_dir[0], ly = cfg.light_dir[1], lz = cfg.light_dir[2];
    const double ln = std::sqrt(lx * lx + ly * ly + lz * lz);
    for (int f = 0; f < 6; ++f) {
        const double lean = ((double)kNormal[f][0] * lx + (double)kNormal[f][1] * ly + (double)kNormal[f][2] * lz) / ln;
        out[f] = (float)((double)cfg.ambient + (lean > 0.0 ? (double)cfg.diffuse * lean : 0.0));
    }
    out[6] = cfg.ambient;
}

// Launch shape of the render kernel: image tiling, strips of tiles per workgroup, the work list per XCD.
static int shape_render(mv::RenderParams& p, const mv_config& cfg, const mv::GridLayout& layout, const mv::LdsPlan& plan,
                        const char* who)
{
    const int num_obs = cfg.num_envs * cfg.agents_per_env;
    p.g = layout;
    p.voxels_per_env = layout.X * layout.Y * layout.Z;
    p.threads = plan.threads;
    p.W = cfg.width; p.H = cfg.height; p.A = cfg.agents_per_env;
    p.materials_plus_one = (cfg.num_materials + 1);
    p.tiles_x = (p.W + mv::kTileW - 1) / mv::kTileW;
    const int tiles_y = (p.H + mv::kTileH - 1) / mv::kTileH;
    p.tiles_per_obs = p.tiles_x * tiles_y;
    int tpb = cfg.tiles_per_block;
    int tpb_tail = 0;                                   // 0: no shorter strips at the end of an XCD's work
    if (tpb <= 0) {
        // Strips of an observation per workgroup.  Two pulls: (1) enough workgroups to fill 256 CUs a few
        // times over (about 6144: on 1024 observations of 40x40x16 worlds, 6 strips per observation render
        // 6 % faster than 8 and 23 % faster than whole observations); (2) when a CU holds four or more
        // workgroups, so that one workgroup's staging hides behind the others' tracing, three strips per
        // observation balance the tail best (40x40x16, 128x72: 3 strips of 48 tiles 5 % faster than 2 on
        // the dynamic workload; 64x64x32 terrain, 256x144, 16 staged layers: 3 strips of 192 tiles 6 %
        // faster than whole observations or 6 strips).  Grids that leave room for only two workgroups per
        // CU render whole observations: every strip would re-stage the rows with nothing to hide it.
        const int waves = p.threads / 64;
        const long long target_blocks = 256ll * 24;
        long long strips = (target_blocks + num_obs - 1) / num_obs;
        if (mv::kLdsBudget / plan.bytes >= 4 && strips < 3) strips = 3;
        if (strips < 1) strips = 1;
        tpb = (int)((p.tiles_per_obs + strips - 1) / strips);
        const int min_tpb = waves * 2;
        if (tpb < min_tpb) tpb = min_tpb;
        // The last twentieth (to tenth, see below) of every XCD's observations is cut into strips a third as long: the XCD's
        // work then ends with short workgroups (4096 x 2 observations, 3 strips of 48 tiles: tail strips of
        // 16 tiles render 1 % faster than none, strips of 24 or 12 tiles gain less; 1024 x 4 observations:
        // 3.6 % faster).
        tpb_tail = tpb / 3;
        if (tpb_tail < min_tpb) tpb_tail = min_tpb;
        if (tpb_tail >= tpb) tpb_tail = 0;
    }
    if (tpb > p.tiles_per_obs) tpb = p.tiles_per_obs;
    p.tiles_per_block = tpb;
    p.blocks_per_obs = (p.tiles_per_obs + tpb - 1) / tpb;
    p.num_obs = num_obs;
    p.obs_per_xcd = (num_obs + mv::kXcds - 1) / mv::kXcds;
    // how much of the range: a twentieth when the launch runs a dozen or more rounds of workgroups through the
    // chip, up to a tenth when it runs only a few (measured optimum on 1024 and 4096 observations: a tenth)
    long long per_cu = (long long)(mv::kLdsBudget / plan.bytes);
    if (per_cu > 32 / (p.threads / 64)) per_cu = 32 / (p.threads / 64);
    if (per_cu < 1) per_cu = 1;
    const long long rounds = (long long)p.blocks_per_obs * num_obs / (256 * per_cu);
    int tail_den = (int)(rounds * 5 / 3);
    if (tail_den < 10) tail_den = 10;
    if (tail_den > 20) tail_den = 20;
    const int tail_obs = tpb_tail > 0 ? p.obs_per_xcd / tail_den : 0;
    p.obs_body_per_xcd = p.obs_per_xcd - tail_obs;
    p.tiles_per_block_tail = tail_obs > 0 ? tpb_tail : tpb;
    p.blocks_per_obs_tail = (p.tiles_per_obs + p.tiles_per_block_tail - 1) / p.tiles_per_block_tail;
    const unsigned long long per_xcd = (unsigned long long)p.obs_body_per_xcd * (unsigned long long)p.blocks_per_obs +
                                       (unsigned long long)tail_obs * (unsigned long long)p.blocks_per_obs_tail;
    if (per_xcd * mv::kXcds > 0x7fffffffull) return fail(MV_ERR_CAPACITY, "%s: too many workgroups", who);
    p.blocks_per_xcd = (uint32_t)per_xcd;
    p.sky_packed = (uint32_t)cfg.sky_rgb[0] | ((uint32_t)cfg.sky_rgb[1] << 8) | ((uint32_t)cfg.sky_rgb[2] << 16);
    p.max_steps = p.g.X + p.g.Y + p.g.Z + 3;
    return MV_OK;
}

extern "C" {

const char* mv_last_error(void) { return g_error; }

void mv_default_config(mv_config* cfg)
{
    if (!cfg) return;
    std::memset(cfg, 0, sizeof(*cfg));
    cfg->width = 128;
    cfg->height = 72;
    cfg->hfov_rad = 1.57079637f;
    cfg->light_dir[0] = 1.0f; cfg->light_dir[1] = 2.0f; cfg->light_dir[2] = 3.0f;
    cfg->ambient = 0.30f;
    cfg->diffuse = 0.70f;
    cfg->sky_rgb[0] = 135; cfg->sky_rgb[1] = 206; cfg->sky_rgb[2] = 235;
}

int mv_create_batch(const mv_config* cfg, mv_batch** out)
{
    if (!cfg || !out) return fail(MV_ERR_ARG, "mv_create_batch: null argument");
    mv::GridLayout layout{};
    mv::LdsPlan plan{};
    {
        const int rc = check_config(cfg, "mv_create_batch", &layout, &plan);
        if (rc != MV_OK) return rc;
    }
    const long long voxels = (long long)cfg->grid_x * cfg->grid_y * cfg->grid_z;
    const long long num_obs = (long long)cfg->num_envs * cfg->agents_per_env;

    int device_count = 0;
    MV_HIP(hipGetDeviceCount(&device_count));
    if (cfg->device >= device_count) return fail(MV_ERR_ARG, "mv_create_batch: device %d of %d", cfg->device, device_count);
    DeviceScope scope(cfg->device);
    if (!scope.ok()) return fail(MV_ERR_HIP, "mv_create_batch: cannot select device %d", cfg->device);

    mv_batch* b = new (std::nothrow) mv_batch;
    if (!b) return fail(MV_ERR_HIP, "mv_create_batch: out of host memory");
    b->cfg = *cfg;
    b->num_obs = (int)num_obs;
    b->voxels_per_env = (int)voxels;
    b->layout = layout;
    b->plan = plan;
    b->materials_plus_one = cfg->num_materials + 1;
    b->tan_half_x = std::tan(0.5 * (double)cfg->hfov_rad);
    b->tan_half_y = b->tan_half_x * (double)cfg->height / (double)cfg->width;
    face_intensities(*cfg, b->intensity);
    b->env_has_grid.assign((size_t)cfg->num_envs, 0);
    b->env_has_palette.assign((size_t)cfg->num_envs, 0);

    const size_t N = (size_t)cfg->num_envs;
    hipError_t e = hipSuccess;
    auto alloc = [&](void** p, size_t bytes) {
        if (e == hipSuccess) e = hipMalloc(p, bytes);
    };
    alloc((void**)&b->d_vox, N * (size_t)voxels);
    alloc((void**)&b->d_bits, N * (size_t)layout.env_words * 8);
    alloc((void**)&b->d_ztop, N * 4);
    alloc((void**)&b->d_palette, N * (size_t)b->materials_plus_one * 3);
    alloc((void**)&b->d_lut, N * (size_t)mv::kNumFaces * b->materials_plus_one * 4);
    alloc((void**)&b->d_sx, (size_t)cfg->width * 4);
    alloc((void**)&b->d_sy, (size_t)cfg->height * 4);
    alloc((void**)&b->d_cams, (size_t)num_obs * 5 * 4);
    alloc((void**)&b->d_self, (size_t)num_obs * 4);
    alloc((void**)&b->d_rec, (size_t)num_obs * sizeof(mv::CameraRecord));
    alloc((void**)&b->d_active, N);
    alloc((void**)&b->d_fraction, (size_t)num_obs * 4);
    alloc((void**)&b->d_overlay_values, (size_t)num_obs * MV_MAX_OVERLAY_VALUES * 4);
    alloc((void**)&b->d_height, 4);
    if (e == hipSuccess) e = hipMemset(b->d_height, 0, 4);
    if (e == hipSuccess) e = hipHostMalloc((void**)&b->h_height, 4, hipHostMallocMapped);
    if (e == hipSuccess) {
        *b->h_height = 0;
        e = hipHostGetDevicePointer((void**)&b->h_height_dev, b->h_height, 0);
    }
    if (e == hipSuccess) e = mv::launch_pixel_scalars(b->d_sx, b->d_sy, cfg->width, cfg->height, nullptr);
    if (e == hipSuccess) e = hipStreamSynchronize(nullptr);
    if (e == hipSuccess) e = mv::prepare_kernels();
    if (e != hipSuccess) {
        free_batch(b);
        return fail(MV_ERR_HIP, "mv_create_batch: device set-up failed: %s", hipGetErrorString(e));
    }
    *out = b;
    return MV_OK;
}

int mv_upload_worlds(mv_batch* b, int32_t first_env, int32_t count, const uint8_t* voxels, const uint8_t* palette,
                     int32_t src_is_device, void* hip_stream)
{
    if (!b || !voxels) return fail(MV_ERR_ARG, "mv_upload_worlds: null argument");
    if (count <= 0) return fail(MV_ERR_ARG, "mv_upload_worlds: count must be positive");
    if (first_env < 0 || first_env > b->cfg.num_envs - count)
        return fail(MV_ERR_RANGE, "mv_upload_worlds: environments %d..%d outside 0..%d", first_env,
                    first_env + count - 1, b->cfg.num_envs - 1);
    if (src_is_device < 0 || src_is_device > MV_SRC_DEVICE_BORROWED)
        return fail(MV_ERR_ARG, "mv_upload_worlds: src_is_device = %d", src_is_device);
    const bool whole = first_env == 0 && count == b->cfg.num_envs;
    if (src_is_device == MV_SRC_DEVICE_BORROWED && !whole)
        return fail(MV_ERR_ARG, "mv_upload_worlds: a borrowed array must hold all %d environments", b->cfg.num_envs);
    if (b->borrowed_vox && !whole)
        return fail(MV_ERR_STATE, "mv_upload_worlds: the batch borrows its material ids; upload all environments to end that");
    DeviceScope scope(b->cfg.device);
    if (!scope.ok()) return fail(MV_ERR_HIP, "mv_upload_worlds: cannot select device %d", b->cfg.device);
    hipStream_t stream = (hipStream_t)hip_stream;
    const size_t V = (size_t)b->voxels_per_env;
    const size_t pal_bytes = (size_t)b->materials_plus_one * 3;
    uint8_t* vox_dst = b->d_vox + (size_t)first_env * V;
    uint8_t* pal_dst = b->d_palette + (size_t)first_env * pal_bytes;
    uint64_t* bits_dst = b->d_bits + (size_t)first_env * b->layout.env_words;
    int32_t* ztop_dst = b->d_ztop + first_env;
    uint32_t* lut_dst = b->d_lut + (size_t)first_env * mv::kNumFaces * b->materials_plus_one;

    if (!src_is_device) {
        const size_t n = (size_t)count * V;
        const uint8_t limit = (uint8_t)b->cfg.num_materials;
        for (size_t i = 0; i < n; ++i)
            if (voxels[i] > limit)
                return fail(MV_ERR_RANGE, "mv_upload_worlds: material id %d at voxel %zu exceeds num_materials %d",
                            (int)voxels[i], i, (int)limit);
        MV_HIP(hipMemcpyAsync(vox_dst, voxels, n, hipMemcpyHostToDevice, stream));
        if (palette) MV_HIP(hipMemcpyAsync(pal_dst, palette, (size_t)count * pal_bytes, hipMemcpyHostToDevice, stream));
        // pageable host memory: make sure the runtime is done reading it before we return
        MV_HIP(hipStreamSynchronize(stream));
        MV_HIP(mv::launch_pack(vox_dst, vox_dst, bits_dst, ztop_dst, count, b->layout, palette ? pal_dst : nullptr,
                               pal_dst, lut_dst, b->materials_plus_one, b->intensity,
                               mv::HeightFeedback{ b->d_height, b->h_height_dev }, stream));
    } else if (src_is_device == MV_SRC_DEVICE_BORROWED) {
        // source and destination of the material copy are the caller's array: nothing is copied
        MV_HIP(mv::launch_pack(voxels, const_cast<uint8_t*>(voxels), bits_dst, ztop_dst, count, b->layout, palette, pal_dst,
                               lut_dst, b->materials_plus_one, b->intensity,
                               mv::HeightFeedback{ b->d_height, b->h_height_dev }, stream));
    } else {
        // one launch: material copy, bit rows, palette copy and colour tables
        MV_HIP(mv::launch_pack(voxels, vox_dst, bits_dst, ztop_dst, count, b->layout, palette, pal_dst, lut_dst,
                               b->materials_plus_one, b->intensity,
                               mv::HeightFeedback{ b->d_height, b->h_height_dev }, stream));
    }
    b->borrowed_vox = src_is_device == MV_SRC_DEVICE_BORROWED ? voxels : nullptr;

    for (int e = first_env; e < first_env + count; ++e) {
        if (!b->env_has_grid[e]) { b->env_has_grid[e] = 1; ++b->envs_with_grid; }
        if (palette && !b->env_has_palette[e]) { b->env_has_palette[e] = 1; ++b->envs_with_palette; }
    }
    return MV_OK;
}

int mv_update_voxels(mv_batch* b, int32_t count, const int32_t* env, const int32_t* voxel_index, const uint8_t* material,
                     int32_t src_is_device, void* hip_stream)
{
    if (!b) return fail(MV_ERR_ARG, "mv_update_voxels: null batch");
    if (count < 0) return fail(MV_ERR_ARG, "mv_update_voxels: negative count");
    if (count == 0) return MV_OK;
    if (!env || !voxel_index || !material) return fail(MV_ERR_ARG, "mv_update_voxels: null argument");
    if (b->borrowed_vox) return fail(MV_ERR_STATE, "mv_update_voxels: the batch borrows its material ids from the caller");
    DeviceScope scope(b->cfg.device);
    if (!scope.ok()) return fail(MV_ERR_HIP, "mv_update_voxels: cannot select device %d", b->cfg.device);
    hipStream_t stream = (hipStream_t)hip_stream;
    const int32_t* d_env = env;
    const int32_t* d_idx = voxel_index;
    const uint8_t* d_mat = material;
    if (!src_is_device) {
        for (int32_t e = 0; e < count; ++e) {
            if (env[e] < 0 || env[e] >= b->cfg.num_envs)
                return fail(MV_ERR_RANGE, "mv_update_voxels: edit %d names environment %d", e, env[e]);
            if (voxel_index[e] < 0 || voxel_index[e] >= b->voxels_per_env)
                return fail(MV_ERR_RANGE, "mv_update_voxels: edit %d names voxel %d", e, voxel_index[e]);
            if (material[e] > b->cfg.num_materials)
                return fail(MV_ERR_RANGE, "mv_update_voxels: edit %d has material id %d > %d", e, (int)material[e],
                            b->cfg.num_materials);
            if (!b->env_has_grid[env[e]])
                return fail(MV_ERR_STATE, "mv_update_voxels: environment %d has no grid yet", env[e]);
        }
        if ((size_t)count > b->edits_capacity) {
            // the staging buffer only ever grows; steady-state steps do not allocate
            size_t cap = b->edits_capacity ? b->edits_capacity : 4096;
            while (cap < (size_t)count) cap *= 2;
            uint8_t* fresh = nullptr;
            MV_HIP(hipMalloc((void**)&fresh, cap * 13));
            MV_HIP(hipStreamSynchronize(stream));
            (void)hipFree(b->d_edits);
            b->d_edits = fresh;
            b->edits_capacity = cap;
        }
        int32_t* s_env = reinterpret_cast<int32_t*>(b->d_edits);
        int32_t* s_idx = s_env + b->edits_capacity;
        uint8_t* s_mat = reinterpret_cast<uint8_t*>(s_idx + b->edits_capacity);
        MV_HIP(hipMemcpyAsync(s_env, env, (size_t)count * 4, hipMemcpyHostToDevice, stream));
        MV_HIP(hipMemcpyAsync(s_idx, voxel_index, (size_t)count * 4, hipMemcpyHostToDevice, stream));
        MV_HIP(hipMemcpyAsync(s_mat, material, (size_t)count, hipMemcpyHostToDevice, stream));
        MV_HIP(hipStreamSynchronize(stream));
        d_env = s_env; d_idx = s_idx; d_mat = s_mat;
    }
    MV_HIP(mv::launch_update_voxels(d_env, d_idx, d_mat, count, b->d_vox, b->d_bits, b->d_ztop, b->cfg.num_envs,
                                    b->voxels_per_env, b->cfg.num_materials, b->layout,
                                    mv::HeightFeedback{ b->d_height, b->h_height_dev }, stream));
    return MV_OK;
}

int mv_move_voxels(mv_batch* b, int32_t count, const int32_t* env, const int32_t* from_voxel, const int32_t* to_voxel,
                   const uint8_t* material, int32_t src_is_device, void* hip_stream)
{
    if (!b) return fail(MV_ERR_ARG, "mv_move_voxels: null batch");
    if (count < 0) return fail(MV_ERR_ARG, "mv_move_voxels: negative count");
    if (count == 0) return MV_OK;
    if (!env || !from_voxel || !to_voxel || !material) return fail(MV_ERR_ARG, "mv_move_voxels: null argument");
    if (b->borrowed_vox) return fail(MV_ERR_STATE, "mv_move_voxels: the batch borrows its material ids from the caller");
    DeviceScope scope(b->cfg.device);
    if (!scope.ok()) return fail(MV_ERR_HIP, "mv_move_voxels: cannot select device %d", b->cfg.device);
    hipStream_t stream = (hipStream_t)hip_stream;
    const int32_t* d_env = env;
    const int32_t* d_from = from_voxel;
    const int32_t* d_to = to_voxel;
    const uint8_t* d_mat = material;
    if (!src_is_device) {
        for (int32_t e = 0; e < count; ++e) {
            if (env[e] < 0 || env[e] >= b->cfg.num_envs)
                return fail(MV_ERR_RANGE, "mv_move_voxels: move %d names environment %d", e, env[e]);
            if (from_voxel[e] < -1 || from_voxel[e] >= b->voxels_per_env || to_voxel[e] < -1 || to_voxel[e] >= b->voxels_per_env)
                return fail(MV_ERR_RANGE, "mv_move_voxels: move %d names voxels %d -> %d", e, from_voxel[e], to_voxel[e]);
            if (material[e] > b->cfg.num_materials)
                return fail(MV_ERR_RANGE, "mv_move_voxels: move %d has material id %d > %d", e, (int)material[e],
                            b->cfg.num_materials);
            if (!b->env_has_grid[env[e]])
                return fail(MV_ERR_STATE, "mv_move_voxels: environment %d has no grid yet", env[e]);
        }
        if ((size_t)count > b->edits_capacity) {
            size_t cap = b->edits_capacity ? b->edits_capacity : 4096;
            while (cap < (size_t)count) cap *= 2;
            uint8_t* fresh = nullptr;
            MV_HIP(hipMalloc((void**)&fresh, cap * 13));
            MV_HIP(hipStreamSynchronize(stream));
            (void)hipFree(b->d_edits);
            b->d_edits = fresh;
            b->edits_capacity = cap;
        }
        int32_t* s_env = reinterpret_cast<int32_t*>(b->d_edits);
        int32_t* s_from = s_env + b->edits_capacity;
        int32_t* s_to = s_from + b->edits_capacity;
        uint8_t* s_mat = reinterpret_cast<uint8_t*>(s_to + b->edits_capacity);
        MV_HIP(hipMemcpyAsync(s_env, env, (size_t)count * 4, hipMemcpyHostToDevice, stream));
        MV_HIP(hipMemcpyAsync(s_from, from_voxel, (size_t)count * 4, hipMemcpyHostToDevice, stream));
        MV_HIP(hipMemcpyAsync(s_to, to_voxel, (size_t)count * 4, hipMemcpyHostToDevice, stream));
        MV_HIP(hipMemcpyAsync(s_mat, material, (size_t)count, hipMemcpyHostToDevice, stream));
        MV_HIP(hipStreamSynchronize(stream));
        d_env = s_env; d_from = s_from; d_to = s_to; d_mat = s_mat;
    }
    MV_HIP(mv::launch_move_voxels(d_env, d_from, d_to, d_mat, count, b->d_vox, b->d_bits, b->d_ztop, b->cfg.num_envs,
                                  b->voxels_per_env, b->cfg.num_materials, b->layout,
                                  mv::HeightFeedback{ b->d_height, b->h_height_dev }, stream));
    return MV_OK;
}

int mv_set_cameras(mv_batch* b, const float* cams, const int32_t* self_voxel, int32_t src_is_device, void* hip_stream)
{
    if (!b || !cams) return fail(MV_ERR_ARG, "mv_set_cameras: null argument");
    DeviceScope scope(b->cfg.device);
    if (!scope.ok()) return fail(MV_ERR_HIP, "mv_set_cameras: cannot select device %d", b->cfg.device);
    hipStream_t stream = (hipStream_t)hip_stream;
    const float* d_cams = cams;
    const int32_t* d_self = self_voxel;
    if (!src_is_device) {
        const size_t n = (size_t)b->num_obs * 5;
        for (size_t i = 0; i < n; ++i)
            if (!std::isfinite(cams[i])) return fail(MV_ERR_ARG, "mv_set_cameras: non-finite value at float %zu", i);
        if (self_voxel)
            for (int o = 0; o < b->num_obs; ++o)
                if (self_voxel[o] < -1 || self_voxel[o] >= b->voxels_per_env)
                    return fail(MV_ERR_RANGE, "mv_set_cameras: self_voxel[%d] = %d outside the grid", o, self_voxel[o]);
        MV_HIP(hipMemcpyAsync(b->d_cams, cams, n * 4, hipMemcpyHostToDevice, stream));
        if (self_voxel) MV_HIP(hipMemcpyAsync(b->d_self, self_voxel, (size_t)b->num_obs * 4, hipMemcpyHostToDevice, stream));
        MV_HIP(hipStreamSynchronize(stream));
        d_cams = b->d_cams;
        d_self = self_voxel ? b->d_self : nullptr;
    }
    MV_HIP(mv::launch_cameras(d_cams, d_self, b->d_rec, b->num_obs, b->tan_half_x, b->tan_half_y,
                              b->cfg.grid_x * b->cfg.grid_y, stream));
    b->cameras_set = true;
    return MV_OK;
}

int mv_render_batch(mv_batch* b, uint8_t* rgb, float* depth, uint8_t* aux_material, int32_t* aux_hit_index,
                    uint8_t* aux_face, void* hip_stream)
{
    if (!b || !rgb || !depth) return fail(MV_ERR_ARG, "mv_render_batch: null argument");
    if ((reinterpret_cast<uintptr_t>(depth) & 3) || (aux_hit_index && (reinterpret_cast<uintptr_t>(aux_hit_index) & 3)))
        return fail(MV_ERR_ARG, "mv_render_batch: depth and aux_hit_index must be 4-byte aligned");
    if (b->envs_with_grid != b->cfg.num_envs || b->envs_with_palette != b->cfg.num_envs)
        return fail(MV_ERR_STATE, "mv_render_batch: %d of %d environments have a grid, %d a palette", b->envs_with_grid,
                    b->cfg.num_envs, b->envs_with_palette);
    if (!b->cameras_set) return fail(MV_ERR_STATE, "mv_render_batch: cameras were never set");
    DeviceScope scope(b->cfg.device);
    if (!scope.ok()) return fail(MV_ERR_HIP, "mv_render_batch: cannot select device %d", b->cfg.device);

    // How many layers of a row-scan grid to stage: as many as the tallest world the kernels have reported
    // so far (read without synchronising: a value that is out of date costs speed, never correctness -- a
    // workgroup whose world is taller than what was staged traces through global memory and reports it),
    // all of them before the first report.
    // A launch that is being captured into a HIP graph will be replayed later, over worlds this call cannot
    // know: it stages every layer (unless the caller fixed the number), so that a replay never falls back to the
    // slow path because the worlds grew after the capture.
    int staged = b->cfg.grid_z;
    if (b->layout.fast) {
        bool capturing = false;
        if (hip_stream) {
            hipStreamCaptureStatus status = hipStreamCaptureStatusNone;
            if (hipStreamIsCapturing((hipStream_t)hip_stream, &status) == hipSuccess)
                capturing = status == hipStreamCaptureStatusActive;
            else
                (void)hipGetLastError();
        }
        if (b->forced_layers > 0) {
            staged = b->forced_layers;
        } else if (!capturing) {
            // one layer above the tallest world: cameras that fly above their world stand in that (empty) layer
            const int seen = *(volatile int32_t*)b->h_height + 1;
            if (seen > 1 && seen < staged) staged = seen;
        }
    }
    const mv::LdsPlan plan = mv::plan_lds(b->layout, b->cfg.width, b->cfg.height, b->materials_plus_one, staged,
                                          b->cfg.coarse_level != 0);

    mv::RenderParams p{};
    p.staged_layers = staged;
    p.coarse_after = b->cfg.coarse_level != 0 ? mv::kCoarseAfterTurns : -1;
    p.heights = mv::HeightFeedback{ b->d_height, b->h_height_dev };
    p.active = b->all_active ? nullptr : b->d_active;
    p.bits = b->d_bits; p.ztop = b->d_ztop; p.vox = b->borrowed_vox ? b->borrowed_vox : b->d_vox; p.lut = b->d_lut; p.rec = b->d_rec; p.sx = b->d_sx; p.sy = b->d_sy;
    p.rgb = rgb; p.depth = depth; p.aux_material = aux_material; p.aux_hit = aux_hit_index; p.aux_face = aux_face;
    {
        const int rc = shape_render(p, b->cfg, b->layout, plan, "mv_render_batch");
        if (rc != MV_OK) return rc;
    }
    MV_HIP(mv::launch_render(p, plan.bytes, (hipStream_t)hip_stream));
    return MV_OK;
}

int mv_set_active(mv_batch* b, const uint8_t* active, int32_t src_is_device, void* hip_stream)
{
    if (!b) return fail(MV_ERR_ARG, "mv_set_active: null batch");
    if (!active) { b->all_active = true; return MV_OK; }
    DeviceScope scope(b->cfg.device);
    if (!scope.ok()) return fail(MV_ERR_HIP, "mv_set_active: cannot select device %d", b->cfg.device);
    hipStream_t stream = (hipStream_t)hip_stream;
    MV_HIP(hipMemcpyAsync(b->d_active, active, (size_t)b->cfg.num_envs,
                          src_is_device ? hipMemcpyDeviceToDevice : hipMemcpyHostToDevice, stream));
    if (!src_is_device) MV_HIP(hipStreamSynchronize(stream));
    b->all_active = false;
    return MV_OK;
}

int mv_draw_bars(mv_batch* b, uint8_t* rgb, const float* fraction, const mv_bar* bar, int32_t src_is_device,
                 void* hip_stream)
{
    if (!b || !rgb || !fraction || !bar) return fail(MV_ERR_ARG, "mv_draw_bars: null argument");
    if (bar->reserved[0] || bar->reserved[1]) return fail(MV_ERR_ARG, "mv_draw_bars: reserved bytes must be 0");
    if (bar->width <= 0 || bar->height <= 0 || bar->x < 0 || bar->y < 0 || bar->x > b->cfg.width - bar->width ||
        bar->y > b->cfg.height - bar->height)
        return fail(MV_ERR_ARG, "mv_draw_bars: bar %dx%d at (%d,%d) does not fit the %dx%d image", bar->width,
                    bar->height, bar->x, bar->y, b->cfg.width, b->cfg.height);
    DeviceScope scope(b->cfg.device);
    if (!scope.ok()) return fail(MV_ERR_HIP, "mv_draw_bars: cannot select device %d", b->cfg.device);
    hipStream_t stream = (hipStream_t)hip_stream;
    const float* d_fraction = fraction;
    if (!src_is_device) {
        for (int o = 0; o < b->num_obs; ++o)
            if (!std::isfinite(fraction[o])) return fail(MV_ERR_ARG, "mv_draw_bars: fraction[%d] is not finite", o);
        MV_HIP(hipMemcpyAsync(b->d_fraction, fraction, (size_t)b->num_obs * 4, hipMemcpyHostToDevice, stream));
        MV_HIP(hipStreamSynchronize(stream));
        d_fraction = b->d_fraction;
    }
    mv::BarParams bp{};
    bp.x = bar->x; bp.y = bar->y; bp.width = bar->width; bp.height = bar->height;
    bp.fill_packed = (uint32_t)bar->fill_rgb[0] | ((uint32_t)bar->fill_rgb[1] << 8) | ((uint32_t)bar->fill_rgb[2] << 16);
    bp.empty_packed = (uint32_t)bar->empty_rgb[0] | ((uint32_t)bar->empty_rgb[1] << 8) | ((uint32_t)bar->empty_rgb[2] << 16);
    MV_HIP(mv::launch_bars(rgb, d_fraction, b->all_active ? nullptr : b->d_active, b->num_obs, b->cfg.agents_per_env,
                           b->cfg.width, b->cfg.height, bp, stream));
    return MV_OK;
}

int mv_draw_overlay(mv_batch* b, uint8_t* rgb, const mv_rect* rects, int32_t num_rects, const float* values,
                    int32_t values_per_obs, int32_t src_is_device, void* hip_stream)
{
    if (!b || !rgb || !rects) return fail(MV_ERR_ARG, "mv_draw_overlay: null argument");
    if (num_rects < 1 || num_rects > MV_MAX_OVERLAY_RECTS)
        return fail(MV_ERR_ARG, "mv_draw_overlay: %d primitives (1..%d)", num_rects, MV_MAX_OVERLAY_RECTS);
    if (values_per_obs < 0 || values_per_obs > MV_MAX_OVERLAY_VALUES)
        return fail(MV_ERR_ARG, "mv_draw_overlay: %d values per observation (0..%d)", values_per_obs, MV_MAX_OVERLAY_VALUES);
    if (!values) values_per_obs = 0;
    mv::OverlayParams op{};
    op.count = num_rects;
    auto packed = [](const uint8_t c[3]) { return (uint32_t)c[0] | ((uint32_t)c[1] << 8) | ((uint32_t)c[2] << 16); };
    for (int k = 0; k < num_rects; ++k) {
        const mv_rect& q = rects[k];
        if (q.width <= 0 || q.height <= 0 || q.x < 0 || q.y < 0 || q.x > b->cfg.width - q.width || q.y > b->cfg.height - q.height)
            return fail(MV_ERR_ARG, "mv_draw_overlay: primitive %d, %dx%d at (%d,%d), does not fit the %dx%d image", k,
                        q.width, q.height, q.x, q.y, b->cfg.width, b->cfg.height);
        if (q.kind != MV_RECT_SOLID && q.kind != MV_RECT_GAUGE_RIGHT && q.kind != MV_RECT_GAUGE_UP)
            return fail(MV_ERR_ARG, "mv_draw_overlay: primitive %d has unknown kind %d", k, (int)q.kind);
        if (q.kind != MV_RECT_SOLID && q.value_index >= values_per_obs)
            return fail(MV_ERR_ARG, "mv_draw_overlay: primitive %d reads value %d of %d", k, (int)q.value_index, values_per_obs);
        mv::OverlayRect& r = op.rect[k];
        r.x = q.x; r.y = q.y; r.width = q.width; r.height = q.height;
        r.front_packed = packed(q.rgb); r.rest_packed = packed(q.rest_rgb);
        r.kind = q.kind; r.value_index = q.value_index;
    }
    DeviceScope scope(b->cfg.device);
    if (!scope.ok()) return fail(MV_ERR_HIP, "mv_draw_overlay: cannot select device %d", b->cfg.device);
    hipStream_t stream = (hipStream_t)hip_stream;
    const float* d_values = values;
    if (values && !src_is_device) {
        const size_t n = (size_t)b->num_obs * (size_t)values_per_obs;
        for (size_t i = 0; i < n; ++i)
            if (!std::isfinite(values[i]))
                return fail(MV_ERR_ARG, "mv_draw_overlay: value %d of observation %d is not finite", (int)(i % values_per_obs),
                            (int)(i / values_per_obs));
        if (n > 0) {
            MV_HIP(hipMemcpyAsync(b->d_overlay_values, values, n * 4, hipMemcpyHostToDevice, stream));
            MV_HIP(hipStreamSynchronize(stream));
        }
        d_values = b->d_overlay_values;
    }
    MV_HIP(mv::launch_overlay(rgb, d_values, values_per_obs, b->all_active ? nullptr : b->d_active, b->num_obs,
                              b->cfg.agents_per_env, b->cfg.width, b->cfg.height, op, stream));
    return MV_OK;
}

int mv_step(mv_batch* b, const mv_step_inputs* in, uint8_t* rgb, float* depth, void* hip_stream)
{
    if (!b || !in || !rgb || !depth) return fail(MV_ERR_ARG, "mv_step: null argument");
    if (in->num_edits < 0) return fail(MV_ERR_ARG, "mv_step: num_edits = %d", in->num_edits);
    if (in->num_edits > 0 && (!in->edit_env || !in->edit_voxel || !in->edit_material))
        return fail(MV_ERR_ARG, "mv_step: %d edits without their arrays", in->num_edits);
    if (!in->cams) return fail(MV_ERR_ARG, "mv_step: cams is null");
    if (in->bar_fraction && !in->bar) return fail(MV_ERR_ARG, "mv_step: bar_fraction without bar");
    if (in->num_overlay < 0 || (in->num_overlay > 0 && !in->overlay))
        return fail(MV_ERR_ARG, "mv_step: %d overlay primitives without their list", in->num_overlay);
    int rc = MV_OK;
    if (in->num_edits > 0)
        rc = mv_update_voxels(b, in->num_edits, in->edit_env, in->edit_voxel, in->edit_material, 1, hip_stream);
    if (rc == MV_OK) rc = mv_set_cameras(b, in->cams, in->self_voxel, 1, hip_stream);
    if (rc == MV_OK) {
        if (in->done) {
            DeviceScope scope(b->cfg.device);
            if (!scope.ok()) return fail(MV_ERR_HIP, "mv_step: cannot select device %d", b->cfg.device);
            MV_HIP(mv::launch_active_from_done(in->done, b->d_active, b->cfg.num_envs, (hipStream_t)hip_stream));
            b->all_active = false;
        } else {
            b->all_active = true;
        }
    }
    if (rc == MV_OK) rc = mv_render_batch(b, rgb, depth, nullptr, nullptr, nullptr, hip_stream);
    if (rc == MV_OK && in->bar_fraction) rc = mv_draw_bars(b, rgb, in->bar_fraction, in->bar, 1, hip_stream);
    if (rc == MV_OK && in->num_overlay > 0)
        rc = mv_draw_overlay(b, rgb, in->overlay, in->num_overlay, in->overlay_values, in->overlay_values_per_obs, 1,
                             hip_stream);
    return rc;
}

int mv_host_alloc(void** out, size_t bytes)
{
    if (!out || bytes == 0) return fail(MV_ERR_ARG, "mv_host_alloc: null pointer or zero size");
    void* ptr = nullptr;
    MV_HIP(hipHostMalloc(&ptr, bytes, hipHostMallocDefault));
    *out = ptr;
    return MV_OK;
}

void mv_host_free(void* ptr)
{
    if (ptr) (void)hipHostFree(ptr);
}

int mv_fetch_observations(mv_batch* b, const uint8_t* rgb_dev, const float* depth_dev, int32_t first_obs, int32_t count,
                          uint8_t* rgb_host, float* depth_host, void* hip_stream)
{
    if (!b) return fail(MV_ERR_ARG, "mv_fetch_observations: null batch");
    if ((rgb_host && !rgb_dev) || (depth_host && !depth_dev))
        return fail(MV_ERR_ARG, "mv_fetch_observations: a host destination needs its device tensor");
    if (count <= 0) return fail(MV_ERR_ARG, "mv_fetch_observations: count must be positive");
    if (first_obs < 0 || first_obs > b->num_obs - count)
        return fail(MV_ERR_RANGE, "mv_fetch_observations: observations %d..%d outside 0..%d", first_obs,
                    first_obs + count - 1, b->num_obs - 1);
    DeviceScope scope(b->cfg.device);
    if (!scope.ok()) return fail(MV_ERR_HIP, "mv_fetch_observations: cannot select device %d", b->cfg.device);
    hipStream_t stream = (hipStream_t)hip_stream;
    const size_t pixels = (size_t)b->cfg.width * (size_t)b->cfg.height;
    if (rgb_host)
        MV_HIP(hipMemcpyAsync(rgb_host, rgb_dev + (size_t)first_obs * pixels * 3, (size_t)count * pixels * 3,
                              hipMemcpyDeviceToHost, stream));
    if (depth_host)
        MV_HIP(hipMemcpyAsync(depth_host, depth_dev + (size_t)first_obs * pixels, (size_t)count * pixels * 4,
                              hipMemcpyDeviceToHost, stream));
    return MV_OK;
}

void mv_destroy(mv_batch* b)
{
    if (!b) return;
    DeviceScope scope(b->cfg.device);
    if (scope.ok()) (void)hipDeviceSynchronize();
    free_batch(b);
}

int mv_debug_occupancy(mv_batch* b, int32_t env, const uint64_t** x_rows, int32_t* x_row_words,
                       const uint64_t** y_rows, int32_t* y_row_words, const int32_t** top_layer)
{
    if (!b || !x_rows || !x_row_words || !y_rows || !y_row_words || !top_layer)
        return fail(MV_ERR_ARG, "mv_debug_occupancy: null argument");
    if (env < 0 || env >= b->cfg.num_envs) return fail(MV_ERR_RANGE, "mv_debug_occupancy: env %d", env);
    *x_rows = b->d_bits + (size_t)env * b->layout.env_words;
    *x_row_words = b->layout.rowwords_x;
    *y_rows = *x_rows + b->layout.xrow_words;
    *y_row_words = b->layout.rowwords_y;
    *top_layer = b->d_ztop + env;
    return MV_OK;
}

int mv_debug_launch_shape(const mv_config* cfg, int32_t staged_layers, mv_launch_shape* shape)
{
    if (!cfg || !shape) return fail(MV_ERR_ARG, "mv_debug_launch_shape: null argument");
    mv::GridLayout layout{};
    mv::LdsPlan plan{};
    const int rc = check_config(cfg, "mv_debug_launch_shape", &layout, &plan);
    if (rc != MV_OK) return rc;
    if (staged_layers < 0 || staged_layers > cfg->grid_z)
        return fail(MV_ERR_RANGE, "mv_debug_launch_shape: %d layers outside 0..%d", staged_layers, cfg->grid_z);
    if (staged_layers > 0)
        plan = mv::plan_lds(layout, cfg->width, cfg->height, cfg->num_materials + 1, staged_layers, cfg->coarse_level != 0);
    mv::RenderParams p{};
    const int rc2 = shape_render(p, *cfg, layout, plan, "mv_debug_launch_shape");
    if (rc2 != MV_OK) return rc2;
    shape->lds_bytes = (int32_t)plan.bytes; shape->threads = plan.threads;
    shape->tiles_x = p.tiles_x; shape->tiles_per_obs = p.tiles_per_obs;
    shape->tiles_per_block = p.tiles_per_block; shape->blocks_per_obs = p.blocks_per_obs;
    shape->tiles_per_block_tail = p.tiles_per_block_tail; shape->blocks_per_obs_tail = p.blocks_per_obs_tail;
    shape->num_obs = p.num_obs; shape->obs_per_xcd = p.obs_per_xcd; shape->obs_body_per_xcd = p.obs_body_per_xcd;
    shape->blocks_per_xcd = p.blocks_per_xcd;
    return MV_OK;
}

int mv_debug_set_staged_layers(mv_batch* b, int32_t layers)
{
    if (!b) return fail(MV_ERR_ARG, "mv_debug_set_staged_layers: null batch");
    if (layers < 0 || layers > b->cfg.grid_z)
        return fail(MV_ERR_RANGE, "mv_debug_set_staged_layers: %d outside 0..%d", layers, b->cfg.grid_z);
    b->forced_layers = layers;
    return MV_OK;
}

int mv_debug_camera_records(mv_batch* b, const void** records)
{
    if (!b || !records) return fail(MV_ERR_ARG, "mv_debug_camera_records: null argument");
    *records = b->d_rec;
    return MV_OK;
}

}  // extern "C"

// ------------------------------------------------------------------------------------------
// mv_render_worlds_noalloc: the whole path for callers that must not allocate.  What a batch object keeps in
// memory from mv_create_batch (bit rows, top layers, colour tables, camera records, pixel scalars) lives in one
// file-scope device array instead; every GPU the library runs on holds its own copy of it until the process
// ends.  In host code the array's name is only a handle for hipGetSymbolAddress: the device address is looked
// up once per device and only that address is ever passed to a kernel.
// ------------------------------------------------------------------------------------------
namespace {

constexpr size_t kScratchBytes = MV_NOALLOC_SCRATCH_BYTES;
constexpr int kScratchDevices = 64;

}  // namespace

static __device__ __align__(256) unsigned char scratch[kScratchBytes];

namespace {

std::mutex g_scratch_mutex;
unsigned char* g_scratch_ptr[kScratchDevices] = {};

// device address of this device's copy of `scratch` (the device must be current)
int scratch_address(int device, unsigned char** out)
{
    if (device < 0 || device >= kScratchDevices)
        return fail(MV_ERR_ARG, "mv_render_worlds_noalloc: device %d outside 0..%d", device, kScratchDevices - 1);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[device]) {
        void* ptr = nullptr;
        MV_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        if (!ptr) return fail(MV_ERR_HIP, "mv_render_worlds_noalloc: no device address for the scratch array");
        g_scratch_ptr[device] = static_cast<unsigned char*>(ptr);
    }
    *out = g_scratch_ptr[device];
    return MV_OK;
}

size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

}  // namespace

extern "C" int mv_render_worlds_noalloc(const mv_config* cfg, const uint8_t* voxels, const uint8_t* palette,
                                        const float* cams, const int32_t* self_voxel, uint8_t* rgb, float* depth,
                                        void* hip_stream)
{
    if (!cfg || !voxels || !palette || !cams || !rgb || !depth)
        return fail(MV_ERR_ARG, "mv_render_worlds_noalloc: null argument");
    if (reinterpret_cast<uintptr_t>(depth) & 3)
        return fail(MV_ERR_ARG, "mv_render_worlds_noalloc: depth must be 4-byte aligned");
    mv::GridLayout layout{};
    mv::LdsPlan plan{};
    {
        const int rc = check_config(cfg, "mv_render_worlds_noalloc", &layout, &plan);
        if (rc != MV_OK) return rc;
    }
    const size_t N = (size_t)cfg->num_envs, NA = N * (size_t)cfg->agents_per_env;
    const int mp1 = cfg->num_materials + 1;
    // carve the scratch array: [bit rows][colour tables][top layers][camera records][sx][sy]
    size_t off = 0;
    const size_t off_bits = off;  off = align256(off + N * (size_t)layout.env_words * 8);
    const size_t off_lut = off;   off = align256(off + N * (size_t)mv::kNumFaces * mp1 * 4);
    const size_t off_ztop = off;  off = align256(off + N * 4);
    const size_t off_rec = off;   off = align256(off + NA * sizeof(mv::CameraRecord));
    const size_t off_sx = off;    off = align256(off + (size_t)cfg->width * 4);
    const size_t off_sy = off;    off = align256(off + (size_t)cfg->height * 4);
    if (off > kScratchBytes)
        return fail(MV_ERR_CAPACITY, "mv_render_worlds_noalloc: %d environments x %d agents of %dx%dx%d voxels need %zu bytes "
                    "of working memory, the fixed scratch array holds %zu; use a batch object (mv_create_batch) instead",
                    cfg->num_envs, cfg->agents_per_env, cfg->grid_x, cfg->grid_y, cfg->grid_z, off, kScratchBytes);

    int device_count = 0;
    MV_HIP(hipGetDeviceCount(&device_count));
    if (cfg->device >= device_count)
        return fail(MV_ERR_ARG, "mv_render_worlds_noalloc: device %d of %d", cfg->device, device_count);
    DeviceScope scope(cfg->device);
    if (!scope.ok()) return fail(MV_ERR_HIP, "mv_render_worlds_noalloc: cannot select device %d", cfg->device);
    unsigned char* base = nullptr;
    {
        const int rc = scratch_address(cfg->device, &base);
        if (rc != MV_OK) return rc;
    }
    MV_HIP(mv::prepare_kernels());
    hipStream_t stream = (hipStream_t)hip_stream;
    uint64_t* d_bits = reinterpret_cast<uint64_t*>(base + off_bits);
    uint32_t* d_lut = reinterpret_cast<uint32_t*>(base + off_lut);
    int32_t* d_ztop = reinterpret_cast<int32_t*>(base + off_ztop);
    mv::CameraRecord* d_rec = reinterpret_cast<mv::CameraRecord*>(base + off_rec);
    float* d_sx = reinterpret_cast<float*>(base + off_sx);
    float* d_sy = reinterpret_cast<float*>(base + off_sy);

    float intensity[mv::kNumFaces];
    face_intensities(*cfg, intensity);
    const double tan_half_x = std::tan(0.5 * (double)cfg->hfov_rad);
    const double tan_half_y = tan_half_x * (double)cfg->height / (double)cfg->width;
    const mv::HeightFeedback no_feedback{ nullptr, nullptr };

    // Every word of the scratch regions used below is rewritten by these launches before the render reads it
    // (pack writes every row word, top layer and table entry of every environment), so nothing left over from an
    // earlier, larger call can show through and nothing needs clearing.
    MV_HIP(mv::launch_pixel_scalars(d_sx, d_sy, cfg->width, cfg->height, stream));
    // source and destination of the material and palette copies are the caller's own arrays: nothing is copied,
    // the render reads the material of a hit voxel from `voxels` directly
    MV_HIP(mv::launch_pack(voxels, const_cast<uint8_t*>(voxels), d_bits, d_ztop, cfg->num_envs, layout, palette,
                           const_cast<uint8_t*>(palette), d_lut, mp1, intensity, no_feedback, stream));
    MV_HIP(mv::launch_cameras(cams, self_voxel, d_rec, (int)NA, tan_half_x, tan_half_y, cfg->grid_x * cfg->grid_y, stream));

    mv::RenderParams p{};
    p.staged_layers = cfg->grid_z;            // no height feedback without a batch object: stage every layer
    p.coarse_after = cfg->coarse_level != 0 ? mv::kCoarseAfterTurns : -1;
    p.heights = no_feedback;
    p.active = nullptr;
    p.bits = d_bits; p.ztop = d_ztop; p.vox = voxels; p.lut = d_lut; p.rec = d_rec; p.sx = d_sx; p.sy = d_sy;
    p.rgb = rgb; p.depth = depth;
    {
        const int rc = shape_render(p, *cfg, layout, plan, "mv_render_worlds_noalloc");
        if (rc != MV_OK) return rc;
    }
    MV_HIP(mv::launch_render(p, plan.bytes, stream));
    return MV_OK;
}
