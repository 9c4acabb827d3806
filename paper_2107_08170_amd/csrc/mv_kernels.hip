// HIP kernels (gfx950 / CDNA4) of the batched voxel-world renderer.
//
// Hot path (paper Sec. 3.2, Eq. 2: O = Render(S), all N*A views in one GPU request):
//   pack      : material ids -> occupancy bits                       (once per world upload)
//   shade     : palette x face intensity -> per-environment colour table
//   cameras   : (x,y,z,yaw,pitch) -> 64-byte camera records (float64 trig, float32 result)
//   render    : one workgroup stages one environment's occupancy bits in LDS; each wave renders
//               8x8-pixel tiles, one pixel ray per lane, 3D-DDA through the bit grid; colour and
//               depth leave as row-major dword stores.
// No MFMA anywhere: nothing on this path is a dense contraction.
#include "mv_internal.h"

#include <math.h>

namespace mv {

// ------------------------------------------------------------------------------------------
// pixel-centre scalars: sx[c] = (2c+1-W)/W, sy[r] = (H-2r-1)/H, one correctly rounded divide each
// ------------------------------------------------------------------------------------------
__global__ void pixel_scalars_kernel(float* __restrict__ sx, float* __restrict__ sy, int W, int H)
{
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < W) sx[i] = __fdiv_rn((float)(2 * i + 1 - W), (float)W);
    if (i < H) sy[i] = __fdiv_rn((float)(H - 2 * i - 1), (float)H);
}

hipError_t launch_pixel_scalars(float* sx, float* sy, int W, int H, hipStream_t stream)
{
    int n = W > H ? W : H;
    hipLaunchKernelGGL(pixel_scalars_kernel, dim3((n + 255) / 256), dim3(256), 0, stream, sx, sy, W, H);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// pack: one thread per 32-voxel word.  Reads 32 material bytes, writes them back to the batch's
// own grid (unless the upload already landed there) and one occupancy word.
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void pack_kernel(const uint8_t* __restrict__ src, uint8_t* __restrict__ vox_dst,
                                                   uint32_t* __restrict__ occ_dst, int voxels_per_env,
                                                   int words_per_env, long long total_words, int vec_ok)
{
    long long gw = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (gw >= total_words) return;
    int env = (int)(gw / words_per_env);
    int w = (int)(gw - (long long)env * words_per_env);
    long long base = (long long)env * voxels_per_env + (long long)w * 32;
    int n = voxels_per_env - w * 32;
    if (n > 32) n = 32;
    uint32_t bits = 0;
    const bool copy = (src != vox_dst);
    if (vec_ok && n == 32) {
        const uint4* s4 = reinterpret_cast<const uint4*>(src + base);
        uint4 a = s4[0], b = s4[1];
        uint32_t v[8] = { a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w };
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            uint32_t x = v[q];
            uint32_t nz = ((x & 0xffu) != 0) | (((x & 0xff00u) != 0) << 1) | (((x & 0xff0000u) != 0) << 2) |
                          (((x & 0xff000000u) != 0) << 3);
            bits |= nz << (4 * q);
        }
        if (copy) {
            uint4* d4 = reinterpret_cast<uint4*>(vox_dst + base);
            d4[0] = a;
            d4[1] = b;
        }
    } else {
        for (int q = 0; q < n; ++q) {
            uint8_t m = src[base + q];
            bits |= (uint32_t)(m != 0) << q;
            if (copy) vox_dst[base + q] = m;
        }
    }
    occ_dst[gw] = bits;
}

hipError_t launch_pack(const uint8_t* src, uint8_t* vox_dst, uint32_t* occ_dst, int count, int voxels_per_env,
                       int words_per_env, hipStream_t stream)
{
    long long total = (long long)count * words_per_env;
    int vec_ok = (voxels_per_env % 32 == 0) && ((reinterpret_cast<uintptr_t>(src) & 15) == 0) &&
                 ((reinterpret_cast<uintptr_t>(vox_dst) & 15) == 0);
    unsigned blocks = (unsigned)((total + 255) / 256);
    hipLaunchKernelGGL(pack_kernel, dim3(blocks), dim3(256), 0, stream, src, vox_dst, occ_dst, voxels_per_env,
                       words_per_env, total, vec_ok);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// shade: lut[env][face][m] = round-to-nearest(palette[env][m] * intensity[face]) per channel,
// two separately rounded float32 operations (multiply, then add 0.5), floor, clamp to 255.
// ------------------------------------------------------------------------------------------
struct Intensities { float v[kNumFaces]; };

__global__ void shade_kernel(const uint8_t* __restrict__ palette, uint32_t* __restrict__ lut, int count,
                             int materials_plus_one, Intensities I)
{
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    int per_env = kNumFaces * materials_plus_one;
    if (i >= count * per_env) return;
    int env = i / per_env;
    int r = i - env * per_env;
    int face = r / materials_plus_one;
    int m = r - face * materials_plus_one;
    const uint8_t* pal = palette + ((size_t)env * materials_plus_one + m) * 3;
    uint32_t packed = 0;
#pragma unroll
    for (int ch = 0; ch < 3; ++ch) {
        float q = floorf(__fadd_rn(__fmul_rn((float)pal[ch], I.v[face]), 0.5f));
        q = fminf(fmaxf(q, 0.0f), 255.0f);
        packed |= (uint32_t)q << (8 * ch);
    }
    lut[i] = packed;
}

hipError_t launch_shade_tables(const uint8_t* palette, uint32_t* lut, int count, int materials_plus_one,
                               const float intensity[kNumFaces], hipStream_t stream)
{
    Intensities I;
    for (int f = 0; f < kNumFaces; ++f) I.v[f] = intensity[f];
    int total = count * kNumFaces * materials_plus_one;
    hipLaunchKernelGGL(shade_kernel, dim3((total + 255) / 256), dim3(256), 0, stream, palette, lut, count,
                       materials_plus_one, I);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// cameras: basis from yaw/pitch in float64, scaled, rounded once to float32.
//   forward F = (cos p cos y, cos p sin y, sin p), right = (sin y, -cos y, 0),
//   up = (-sin p cos y, -sin p sin y, cos p)
// ------------------------------------------------------------------------------------------
__global__ void camera_kernel(const float* __restrict__ cams, const int32_t* __restrict__ self_voxel,
                              CameraRecord* __restrict__ rec, int num_obs, double tan_half_x, double tan_half_y,
                              int plane_voxels)
{
    int o = blockIdx.x * blockDim.x + threadIdx.x;
    if (o >= num_obs) return;
    const float* c = cams + 5 * (size_t)o;
    double yaw = (double)c[3], pitch = (double)c[4];
    double sy, cy, sp, cp;
    sincos(yaw, &sy, &cy);
    sincos(pitch, &sp, &cp);
    CameraRecord r;
    r.P[0] = c[0]; r.P[1] = c[1]; r.P[2] = c[2];
    r.F[0] = (float)(cp * cy); r.F[1] = (float)(cp * sy); r.F[2] = (float)sp;
    r.R[0] = (float)(tan_half_x * sy); r.R[1] = (float)(tan_half_x * -cy); r.R[2] = (float)(tan_half_x * 0.0);
    r.U[0] = (float)(tan_half_y * (-sp * cy)); r.U[1] = (float)(tan_half_y * (-sp * sy)); r.U[2] = (float)(tan_half_y * cp);
    int s = self_voxel ? self_voxel[o] : -1;
    r.self_lo = s >= 0 ? s : -1;
    r.self_hi = s >= 0 ? s + plane_voxels : -1;
    r.pad[0] = r.pad[1] = 0;
    rec[o] = r;
}

hipError_t launch_cameras(const float* cams, const int32_t* self_voxel, CameraRecord* rec, int num_obs,
                          double tan_half_x, double tan_half_y, int plane_voxels, hipStream_t stream)
{
    hipLaunchKernelGGL(camera_kernel, dim3((num_obs + 127) / 128), dim3(128), 0, stream, cams, self_voxel, rec,
                       num_obs, tan_half_x, tan_half_y, plane_voxels);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// render
// ------------------------------------------------------------------------------------------
struct Hit {
    int   idx;      // linear voxel index, -1 = miss
    int   face;     // 0..6, 255 = miss
    float t;        // planar depth
};

// One ray through the LDS-resident bit grid.  Crossing parameters are recomputed as
// t = n*|1/d| + t_first (one fused op, error relative to t itself) rather than accumulated, so the
// position error at any crossing stays a few 1e-6 voxels across the whole grid.
template <bool HAS_SELF>
__device__ __forceinline__ Hit trace_ray(const uint32_t* __restrict__ occ, const float P[3], const float d[3],
                                         int X, int Y, int Z, bool origin_in_grid, int self_lo, int self_hi,
                                         int max_steps)
{
    const float kInf = __builtin_inff();
    const int dim[3] = { X, Y, Z };
    Hit miss = { -1, 255, 0.0f };

    float inv[3];
    bool pos[3], zero[3];
#pragma unroll
    for (int a = 0; a < 3; ++a) {
        zero[a] = d[a] == 0.0f;
        pos[a] = d[a] > 0.0f;
        inv[a] = zero[a] ? 0.0f : __builtin_amdgcn_rcpf(d[a]);
    }

    float t0 = 0.0f;
    int entry_axis = -1;
    if (!origin_in_grid) {                       // wave-uniform: the camera is the same for the tile
        float t_near = -kInf, t_far = kInf;
        bool dead = false;
#pragma unroll
        for (int a = 0; a < 3; ++a) {
            if (zero[a]) {
                dead |= (P[a] < 0.0f) | (P[a] > (float)dim[a]);
            } else {
                float ta = ((pos[a] ? 0.0f : (float)dim[a]) - P[a]) * inv[a];
                float tb = ((pos[a] ? (float)dim[a] : 0.0f) - P[a]) * inv[a];
                if (ta > t_near) { t_near = ta; entry_axis = a; }
                t_far = fminf(t_far, tb);
            }
        }
        if (dead || t_near > t_far || t_far < 0.0f) return miss;
        if (t_near > 0.0f) t0 = t_near; else entry_axis = -1;
    }

    int cell[3];
    float t_next[3], t_first[3], dt[3], n[3];
    int stride[3] = { 1, X, X * Y };
    float t_exit = kInf;                          // parameter at which the ray leaves the grid box
#pragma unroll
    for (int a = 0; a < 3; ++a) {
        float q = floorf(fmaf(t0, d[a], P[a]));
        int c = (int)fminf(fmaxf(q, 0.0f), (float)(dim[a] - 1));
        if (a == entry_axis) c = pos[a] ? 0 : dim[a] - 1;
        cell[a] = c;
        float plane = (float)(c + (pos[a] ? 1 : 0));
        t_first[a] = zero[a] ? kInf : (plane - P[a]) * inv[a];
        dt[a] = fabsf(inv[a]);
        n[a] = 0.0f;
        t_next[a] = t_first[a];
        // number of planes between the current cell and the outside of the grid, this axis
        float planes_left = (float)(pos[a] ? dim[a] - 1 - c : c);
        float te = zero[a] ? kInf : fmaf(planes_left, dt[a], t_first[a]);
        t_exit = fminf(t_exit, te);
        if (!pos[a]) stride[a] = -stride[a];
    }

    int idx = (cell[2] * Y + cell[1]) * X + cell[0];
    float t_hit = t0;
    int face = entry_axis >= 0 ? 2 * entry_axis + (pos[entry_axis] ? 0 : 1) : 6;

    auto solid = [&](int i) -> bool {
        bool s = (occ[i >> 5] >> (i & 31)) & 1u;
        if (HAS_SELF) s = s && i != self_lo && i != self_hi;
        return s;
    };
    if (solid(idx)) return Hit{ idx, face, t_hit };

    for (int it = 0; it < max_steps; ++it) {
        float tm = fminf(fminf(t_next[0], t_next[1]), t_next[2]);
        // leaving the grid: the exit parameter was built from the same n*dt+t_first expression, so
        // this comparison is exact
        if (!(tm < t_exit)) return miss;
        bool cx = (t_next[0] <= t_next[1]) & (t_next[0] <= t_next[2]);
        bool cy = !cx & (t_next[1] <= t_next[2]);
        bool cz = !cx & !cy;
        n[0] += cx ? 1.0f : 0.0f;
        n[1] += cy ? 1.0f : 0.0f;
        n[2] += cz ? 1.0f : 0.0f;
        idx += cx ? stride[0] : (cy ? stride[1] : stride[2]);
        t_next[0] = fmaf(n[0], dt[0], t_first[0]);
        t_next[1] = fmaf(n[1], dt[1], t_first[1]);
        t_next[2] = fmaf(n[2], dt[2], t_first[2]);
        if (solid(idx)) {
            int axis = cx ? 0 : (cy ? 1 : 2);
            bool p = cx ? pos[0] : (cy ? pos[1] : pos[2]);
            return Hit{ idx, 2 * axis + (p ? 0 : 1), tm };
        }
    }
    return miss;
}

template <bool AUX, bool PACKED>
__global__ __launch_bounds__(kBlockThreads) void render_kernel(RenderParams p)
{
    extern __shared__ uint32_t lds_occ[];

    // XCD-aware mapping: hardware deals workgroup b to XCD b % 8; give each XCD a contiguous range
    // of work items so that the blocks sharing an environment also share an L2.
    const uint32_t b = blockIdx.x;
    const uint32_t work = (b % kXcds) * p.blocks_per_xcd + b / kXcds;
    if (work >= p.total_blocks) return;
    const int obs = (int)(work / (uint32_t)p.blocks_per_obs);
    const int part = (int)(work - (uint32_t)obs * (uint32_t)p.blocks_per_obs);
    const int env = obs / p.A;

    {   // a3: stage this environment's occupancy bits
        const uint32_t* g = p.occ + (size_t)env * p.words_per_env;
        if ((p.words_per_env & 3) == 0) {
            const uint4* g4 = reinterpret_cast<const uint4*>(g);
            uint4* l4 = reinterpret_cast<uint4*>(lds_occ);
            for (int w = threadIdx.x; w < (p.words_per_env >> 2); w += kBlockThreads) l4[w] = g4[w];
        } else {
            for (int w = threadIdx.x; w < p.words_per_env; w += kBlockThreads) lds_occ[w] = g[w];
        }
    }
    __syncthreads();

    const CameraRecord& rec = p.rec[obs];
    const float P[3] = { rec.P[0], rec.P[1], rec.P[2] };
    const int self_lo = rec.self_lo, self_hi = rec.self_hi;
    const bool origin_in_grid = P[0] >= 0.0f && P[0] <= (float)p.X && P[1] >= 0.0f && P[1] <= (float)p.Y &&
                                P[2] >= 0.0f && P[2] <= (float)p.Z;

    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    const int tile_begin = part * p.tiles_per_block;
    const int tile_end = min(tile_begin + p.tiles_per_block, p.tiles_per_obs);
    const size_t obs_pix = (size_t)obs * p.H * p.W;

    for (int tile = tile_begin + wave; tile < tile_end; tile += kWavesPerBlock) {
        const int ty = tile / p.tiles_x, tx = tile - ty * p.tiles_x;
        const int col = tx * kTile + (lane & 7), row = ty * kTile + (lane >> 3);
        const bool active = col < p.W && row < p.H;
        const int ccol = min(col, p.W - 1), crow = min(row, p.H - 1);

        // a4: ray through the pixel centre, two fused multiply-adds per axis
        const float sx = p.sx[ccol], sy = p.sy[crow];
        float d[3];
#pragma unroll
        for (int a = 0; a < 3; ++a) d[a] = fmaf(sy, rec.U[a], fmaf(sx, rec.R[a], rec.F[a]));

        // a5: traversal
        Hit h = (self_lo >= 0)
                    ? trace_ray<true>(lds_occ, P, d, p.X, p.Y, p.Z, origin_in_grid, self_lo, self_hi, p.max_steps)
                    : trace_ray<false>(lds_occ, P, d, p.X, p.Y, p.Z, origin_in_grid, -1, -1, p.max_steps);

        // a6: shade
        uint32_t colour = p.sky_packed;
        int material = 0;
        if (h.idx >= 0) {
            material = p.vox[(size_t)env * p.voxels_per_env + h.idx];
            int m = min(material, p.materials_plus_one - 1);
            colour = p.lut[((size_t)env * kNumFaces + h.face) * p.materials_plus_one + m];
        }

        // a7: stores
        const size_t pix = obs_pix + (size_t)crow * p.W + ccol;
        if (active) {
            p.depth[pix] = h.t;
            if (AUX) {
                if (p.aux_material) p.aux_material[pix] = (uint8_t)material;
                if (p.aux_hit) p.aux_hit[pix] = h.idx;
                if (p.aux_face) p.aux_face[pix] = (uint8_t)h.face;
            }
        }
        if (PACKED) {
            // W % 4 == 0: four consecutive lanes hold four consecutive pixels of one row = 12 bytes =
            // three aligned dwords, written by the first three lanes of the quad.
            const uint32_t next = __shfl_down(colour, 1);
            const int m = lane & 3;
            const uint32_t word = (colour >> (8 * m)) | (next << (24 - 8 * m));
            if (active && m < 3) {
                uint32_t* out = reinterpret_cast<uint32_t*>(p.rgb + (pix - m) * 3) + m;
                *out = word;
            }
        } else if (active) {
            uint8_t* out = p.rgb + pix * 3;
            out[0] = (uint8_t)colour;
            out[1] = (uint8_t)(colour >> 8);
            out[2] = (uint8_t)(colour >> 16);
        }
    }
}

size_t render_lds_bytes(int words_per_env)
{
    return ((size_t)words_per_env * 4 + 15) & ~(size_t)15;
}

hipError_t launch_render(const RenderParams& p, size_t lds_bytes, hipStream_t stream)
{
    const bool aux = p.aux_material || p.aux_hit || p.aux_face;
    const bool packed = (p.W % 4 == 0) && ((reinterpret_cast<uintptr_t>(p.rgb) & 3) == 0);
    dim3 grid(p.blocks_per_xcd * kXcds), block(kBlockThreads);
    if (aux) {
        if (packed) hipLaunchKernelGGL((render_kernel<true, true>), grid, block, lds_bytes, stream, p);
        else        hipLaunchKernelGGL((render_kernel<true, false>), grid, block, lds_bytes, stream, p);
    } else {
        if (packed) hipLaunchKernelGGL((render_kernel<false, true>), grid, block, lds_bytes, stream, p);
        else        hipLaunchKernelGGL((render_kernel<false, false>), grid, block, lds_bytes, stream, p);
    }
    return hipGetLastError();
}

}  // namespace mv
