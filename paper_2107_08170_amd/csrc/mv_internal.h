// Internal declarations shared by the host runtime (mv_host.hip) and the kernels
// (mv_kernels.hip) of the MI355X batched voxel-world renderer.  Not part of the public ABI.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mv {

// One camera, 64 bytes: position, forward axis, right axis scaled by tan(hfov/2), up axis scaled
// by tan(hfov/2)*H/W, and the two voxels of the camera's own body (-1 = none).
struct alignas(64) CameraRecord {
    float   P[3], F[3], R[3], U[3];
    int32_t self_lo, self_hi;
    int32_t pad[2];
};
static_assert(sizeof(CameraRecord) == 64, "camera record must be 64 bytes");

// A wave renders a tile of kTileW x kTileH = 64 pixels.  8 x 8 keeps the rays of a wave most alike; 16 x 4 would
// halve the row segments a store touches but costs more turns of the row loop (+1.8 % measured), 32 x 2 +8 %.
constexpr int kTileW = 8;
constexpr int kTileH = 64 / kTileW;
static_assert(kTileW * kTileH == 64 && kTileW % 4 == 0, "tile shape");
constexpr int kXcds = 8;                  // MI355X: 8 XCDs, workgroups are dealt round-robin
constexpr int kNumFaces = 7;              // six faces + "inside"
constexpr size_t kLdsBudget = 160 * 1024; // LDS one workgroup may use on gfx950
constexpr int kCoarseAfterTurns = 5;       // coarse level: ordinary turns of a ray before it starts looking at pairs of rows
constexpr size_t kPackStaticLds = 1024;   // room kept for the pack kernel's static LDS words next to its dynamic share

// Occupancy bits in device memory, per environment ("bit rows"):
//   x rows: Z*Y rows of rowwords_x 64-bit words; row (k*Y + j), bit i   <-> voxel (i,j,k)
//   y rows: Z*X rows of rowwords_y 64-bit words; row (k*X + i), bit j   <-> voxel (i,j,k)
// A ray mostly along x scans x rows, one mostly along y scans y rows: a whole run of cells along
// the row is tested with one shift, instead of one DDA step per cell.
struct GridLayout {
    int32_t X, Y, Z;
    int32_t rowwords_x, rowwords_y;       // 64-bit words per row
    int32_t xrow_words, yrow_words;       // 64-bit words of the x-row / y-row arrays of one environment
    int32_t env_words;                    // xrow_words + yrow_words
    int32_t fast;                         // 1: X,Y <= 64 (one word per row) -> row-scan traversal
};

// The tallest world a batch has held so far (1 + highest solid layer over all environments, never
// lowered): `device_max` is exact; `host_max` is a word of pinned host memory that kernels update when the
// device word rises and that the host reads WITHOUT synchronising to decide how many layers the next
// render stages in LDS.  A stale value costs speed only: workgroups that need more layers than were staged
// trace through the rows in global memory instead, and report what they needed.
struct HeightFeedback {
    int32_t* device_max;
    int32_t* host_max;      // device-visible address of the pinned host word
};

struct RenderParams {
    const uint64_t*     bits;             // [N][env_words]
    const int32_t*      ztop;             // [N] 1 + highest solid layer (0 = empty world)
    const uint8_t*      vox;              // [N][V] material ids
    const uint32_t*     lut;              // [N][7][M+1] shaded colours, r | g<<8 | b<<16
    const CameraRecord* rec;              // [N*A]
    const uint8_t*      active;           // [N] non-zero = render, or nullptr = all
    const float*        sx;               // [W] pixel-centre scalars, (2c+1-W)/W
    const float*        sy;               // [H] (H-2r-1)/H
    uint8_t*            rgb;              // [N*A][H][W][3]
    float*              depth;            // [N*A][H][W]
    uint8_t*            aux_material;     // or nullptr
    int32_t*            aux_hit;          // or nullptr
    uint8_t*            aux_face;         // or nullptr
    GridLayout g;
    int32_t voxels_per_env;
    int32_t W, H, A;
    int32_t materials_plus_one;
    int32_t tiles_x, tiles_per_obs;
    // Work list: each XCD renders a contiguous range of obs_per_xcd observations, one workgroup per strip of
    // tiles_per_block tiles; the last observations of the range (from obs_body_per_xcd on) are cut into
    // shorter strips of tiles_per_block_tail tiles so that the XCD's last workgroups are short ones.
    int32_t tiles_per_block, blocks_per_obs, tiles_per_block_tail, blocks_per_obs_tail;
    int32_t num_obs, obs_per_xcd, obs_body_per_xcd;
    uint32_t blocks_per_xcd;
    uint32_t sky_packed;
    int32_t max_steps;
    int32_t threads;                      // workgroup size (multiple of 64)
    int32_t staged_layers;                // row-scan grids: layers 0 .. staged_layers-1 of the bit rows go to LDS
    int32_t coarse_after;                 // < 0: no coarse level; else the ordinary turns a ray makes before it uses it
    HeightFeedback heights;
};

GridLayout make_layout(int X, int Y, int Z);

// LDS plan of the render kernel for a batch; returns 0 if the grid cannot be staged at all.
struct LdsPlan {
    size_t bytes;         // dynamic LDS per workgroup
    int    threads;       // workgroup size that keeps a CU busy with that much LDS
};
// staged_layers: how many z layers of a row-scan grid the workgroup keeps in LDS (1..Z; ignored for other grids);
// coarse: with the pair-of-rows arrays of the optional coarse level
LdsPlan plan_lds(const GridLayout& g, int W, int H, int materials_plus_one, int staged_layers, bool coarse);

// Launchers (mv_kernels.hip).  All enqueue on `stream` and return hipGetLastError().
hipError_t launch_pixel_scalars(float* sx, float* sy, int W, int H, hipStream_t stream);
// pal_src == nullptr keeps the palettes; otherwise [count][M+1][3] device bytes (may equal pal_dst)
hipError_t launch_pack(const uint8_t* src, uint8_t* vox_dst, uint64_t* bits_dst, int32_t* ztop_dst, int count,
                       const GridLayout& g, const uint8_t* pal_src, uint8_t* pal_dst, uint32_t* lut_dst,
                       int materials_plus_one, const float intensity[kNumFaces], const HeightFeedback& heights,
                       hipStream_t stream);
hipError_t launch_update_voxels(const int32_t* env, const int32_t* voxel_index, const uint8_t* material, int count,
                                uint8_t* vox, uint64_t* bits, int32_t* ztop, int num_envs, int voxels_per_env,
                                int num_materials, const GridLayout& g, const HeightFeedback& heights,
                                hipStream_t stream);
hipError_t launch_move_voxels(const int32_t* env, const int32_t* from_voxel, const int32_t* to_voxel,
                              const uint8_t* material, int count, uint8_t* vox, uint64_t* bits, int32_t* ztop,
                              int num_envs, int voxels_per_env, int num_materials, const GridLayout& g,
                              const HeightFeedback& heights, hipStream_t stream);
hipError_t launch_cameras(const float* cams, const int32_t* self_voxel, CameraRecord* rec, int num_obs,
                          double tan_half_x, double tan_half_y, int plane_voxels, hipStream_t stream);
struct BarParams {
    int32_t x, y, width, height;
    uint32_t fill_packed, empty_packed;   // r | g<<8 | b<<16
};
hipError_t launch_bars(uint8_t* rgb, const float* fraction, const uint8_t* active, int num_obs, int A, int W, int H,
                       const BarParams& bar, hipStream_t stream);
// overlay primitives, passed to the kernel by value (kind: 0 solid, 1 gauge to the right, 2 gauge upwards)
constexpr int kMaxOverlayRects = 32;
struct OverlayRect {
    int32_t x, y, width, height;
    uint32_t front_packed, rest_packed;   // r | g<<8 | b<<16
    int32_t kind, value_index;
};
struct OverlayParams {
    int32_t count;
    OverlayRect rect[kMaxOverlayRects];
};
hipError_t launch_overlay(uint8_t* rgb, const float* values, int values_per_obs, const uint8_t* active, int num_obs, int A,
                          int W, int H, const OverlayParams& overlay, hipStream_t stream);
// active[i] = (done[i] == 0) for the n environments of a batch
hipError_t launch_active_from_done(const uint8_t* done, uint8_t* active, int n, hipStream_t stream);
// raises the dynamic-LDS limit of the render and pack kernels on the current device (cheap after the first call)
hipError_t prepare_kernels();
// dynamic LDS the pack kernel asks for: one z layer per wave
size_t pack_lds_bytes(const GridLayout& g);
hipError_t launch_render(const RenderParams& p, size_t lds_bytes, hipStream_t stream);

}  // namespace mv
