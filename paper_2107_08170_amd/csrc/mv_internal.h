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

constexpr int kBlockThreads = 256;        // 4 wave64
constexpr int kWavesPerBlock = kBlockThreads / 64;
constexpr int kTile = 8;                  // a wave renders an 8x8 pixel tile
constexpr int kXcds = 8;                  // MI355X: 8 XCDs, workgroups are dealt round-robin
constexpr int kNumFaces = 7;              // six faces + "inside"

struct RenderParams {
    const uint32_t*     occ;              // [N][words_per_env] occupancy bits, bit = linear voxel index
    const uint8_t*      vox;              // [N][V] material ids
    const uint32_t*     lut;              // [N][7][M+1] shaded colours, r | g<<8 | b<<16
    const CameraRecord* rec;              // [N*A]
    const float*        sx;               // [W] pixel-centre scalars, (2c+1-W)/W
    const float*        sy;               // [H] (H-2r-1)/H
    uint8_t*            rgb;              // [N*A][H][W][3]
    float*              depth;            // [N*A][H][W]
    uint8_t*            aux_material;     // or nullptr
    int32_t*            aux_hit;          // or nullptr
    uint8_t*            aux_face;         // or nullptr
    int32_t words_per_env;
    int32_t voxels_per_env;
    int32_t X, Y, Z, W, H, A;
    int32_t materials_plus_one;
    int32_t tiles_x, tiles_per_obs, tiles_per_block, blocks_per_obs;
    uint32_t total_blocks, blocks_per_xcd;
    uint32_t sky_packed;
    int32_t max_steps;
};

// Launchers (mv_kernels.hip).  All enqueue on `stream` and return hipGetLastError().
hipError_t launch_pixel_scalars(float* sx, float* sy, int W, int H, hipStream_t stream);
hipError_t launch_pack(const uint8_t* src, uint8_t* vox_dst, uint32_t* occ_dst, int count,
                       int voxels_per_env, int words_per_env, hipStream_t stream);
hipError_t launch_shade_tables(const uint8_t* palette, uint32_t* lut, int count, int materials_plus_one,
                               const float intensity[kNumFaces], hipStream_t stream);
hipError_t launch_cameras(const float* cams, const int32_t* self_voxel, CameraRecord* rec, int num_obs,
                          double tan_half_x, double tan_half_y, int plane_voxels, hipStream_t stream);
hipError_t launch_render(const RenderParams& p, size_t lds_bytes, hipStream_t stream);
size_t render_lds_bytes(int words_per_env);

}  // namespace mv
