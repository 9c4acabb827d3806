// HIP kernels (gfx950 / CDNA4) of the batched voxel-world renderer.
//
// Hot path (paper Sec. 3.2, Eq. 2: O = Render(S), all N*A views in one GPU request):
//   pack      : material ids -> occupancy "bit rows" along x and along y, and palette x face intensity ->
//               per-environment colour table (once per world upload)
//   cameras   : (x,y,z,yaw,pitch) -> 64-byte camera records (float64 trig, float32 result)
//   render    : a workgroup stages one environment's bit rows in LDS (plus mirrored copies, so that
//               every ray scans towards increasing bit positions); each wave renders 8x8-pixel
//               tiles, one pixel ray per lane.  The traversal is a DDA over the (v,z) rows the ray
//               passes through, where u is the ray's dominant horizontal axis: all cells the ray
//               covers inside one row are tested with a single 64-bit shift.  Colour and depth
//               leave as row-major dword stores.
// No MFMA anywhere: nothing on this path is a dense contraction.
#include "mv_internal.h"

#include <math.h>
#include <atomic>
#include <type_traits>

namespace mv {

// ------------------------------------------------------------------------------------------
// layout helpers (host)
// ------------------------------------------------------------------------------------------
GridLayout make_layout(int X, int Y, int Z)
{
    GridLayout g{};
    g.X = X; g.Y = Y; g.Z = Z;
    g.rowwords_x = (X + 63) / 64;
    g.rowwords_y = (Y + 63) / 64;
    g.xrow_words = Z * Y * g.rowwords_x;
    g.yrow_words = Z * X * g.rowwords_y;
    g.env_words = g.xrow_words + g.yrow_words;
    g.fast = (X <= 64 && Y <= 64) ? 1 : 0;
    return g;
}

constexpr int kScanClasses = 16;        // (dominant axis) x (direction along u, v, z)
// bytes between scan-class records in LDS (80 used, 16 more with the coarse level): 28 dwords, so that the sixteen
// records start in sixteen different banks (a tile whose rays fall into several classes reads several records at
// once; 128 bytes apart they collided: render +0.6 %)
constexpr int kClassStride = 112;

static size_t align16(size_t v) { return (v + 15) & ~(size_t)15; }

// LDS map (bytes):  [16 scan-class records, 112 B apart] | [sx: W floats][one RowRecord per image row] |
//                   [colour table 7*(M+1) dwords] | bit rows
// fast grids stage four row arrays (x, x mirrored, y, y mirrored) of `staged_layers` layers each; others stage
// all x rows.  With the coarse level, four more arrays follow: the OR of each pair of neighbouring rows of a layer.
struct LdsMap {
    uint32_t scalars, classes, lut, rows;
    uint32_t total;
};

static LdsMap lds_map(const GridLayout& g, int W, int H, int materials_plus_one, int staged_layers, bool coarse)
{
    LdsMap m{};
    size_t off = 0;
    m.classes = (uint32_t)off; off += kScanClasses * kClassStride;
    m.scalars = (uint32_t)off; off = align16(off + (size_t)W * 4) + (size_t)H * 16;      // sx[W], then a 16-byte record per image row
    m.lut = (uint32_t)off;
    off = align16(off + (size_t)kNumFaces * materials_plus_one * 4);
    m.rows = (uint32_t)off;
    off += g.fast ? 16 * (size_t)staged_layers * (size_t)(g.X + g.Y) : (size_t)g.xrow_words * 8;
    if (g.fast && coarse) off += 16 * (size_t)staged_layers * (size_t)((g.X + 1) / 2 + (g.Y + 1) / 2);
    m.total = (uint32_t)off;
    return m;
}

LdsPlan plan_lds(const GridLayout& g, int W, int H, int materials_plus_one, int staged_layers, bool coarse)
{
    LdsPlan plan{};
    const LdsMap m = lds_map(g, W, H, materials_plus_one, staged_layers, coarse);
    if (m.total > kLdsBudget) return plan;                                  // bytes == 0: does not fit
    plan.bytes = m.total;
    // as many waves per workgroup as fill the CU's wave slots with the workgroups its LDS can hold
    // (measured: 64x64x32 grids, two workgroups per CU: 1024 threads render 9 % faster than 512)
    size_t per_cu = kLdsBudget / plan.bytes;
    size_t waves = 32 / (per_cu < 1 ? 1 : per_cu);          // 32 wave slots per CU
    waves &= ~(size_t)3;                                    // whole multiples of the 4 SIMDs: 5 or 6 waves per
    if (waves < 4) waves = 4;                               // workgroup load the SIMDs unevenly (-10 % measured)
    if (waves > 16) waves = 16;
    plan.threads = (int)(waves * 64);
    return plan;
}

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
// pack: one workgroup per environment.  Each wave takes whole z layers: the layer's material bytes
// are prefetched into registers one layer ahead, go through LDS and leave again as the batch's own
// copy.  Grids of one word per row (X, Y <= 64, X a multiple of 4): lane j turns x row j into bits
// dword by dword (non-zero bytes -> nibble with a carry trick and one dot product), and the y rows
// are the 64x64 bit transpose of the x rows, done across lanes without memory.  Other grids: lane r
// gathers row r cell by cell.  Rows leave as one coalesced store per 64 rows.
// A layer of air (no byte set) skips LDS and the transpose: its rows are written as zero words.
// ------------------------------------------------------------------------------------------
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kPackThreads = 256;

// Colour table entry (a6): round-to-nearest(palette value * face intensity) per channel as two
// separately rounded float32 operations (multiply, then add 0.5), floor, clamp to 255; r | g<<8 | b<<16.
struct Intensities { float v[kNumFaces]; };

__device__ __forceinline__ uint32_t shade_entry(const uint8_t* rgb, float intensity)
{
    uint32_t packed = 0;
#pragma unroll
    for (int ch = 0; ch < 3; ++ch) {
        float q = floorf(__fadd_rn(__fmul_rn((float)rgb[ch], intensity), 0.5f));
        q = fminf(fmaxf(q, 0.0f), 255.0f);
        packed |= (uint32_t)q << (8 * ch);
    }
    return packed;
}

// 1 if the byte is non-zero (one v_min_u32; written as asm because the compiler otherwise expands the
// idiom into a compare and a select)
__device__ __forceinline__ uint32_t nonzero(uint32_t byte)
{
    uint32_t r;
    asm("v_min_u32 %0, 1, %1" : "=v"(r) : "v"(byte));
    return r;
}

// Bits of `count` cells starting at `cell`, `stride` bytes apart: bit b = (cell[b*stride] != 0).
__device__ __forceinline__ uint64_t gather_row_bits(const uint8_t* cell, int stride, int count)
{
    uint32_t lo = 0, hi = 0;
    const int n_lo = min(count, 32);
    // unrolled so that the LDS reads of several cells are in flight together
#pragma unroll 8
    for (int b = 0; b < n_lo; ++b) lo |= nonzero(cell[b * stride]) << b;
#pragma unroll 8
    for (int b = 32; b < count; ++b) hi |= nonzero(cell[b * stride]) << (b - 32);
    return ((uint64_t)hi << 32) | lo;
}

// 64x64 bit-matrix transpose across the wave: on entry lane j holds row j, on return lane i holds
// column i (bit j of the result = bit i of lane j's input).  Recursive block swap: at distance S
// lanes l and l^S exchange the off-diagonal SxS blocks.  The partner's word comes over the LDS
// crossbar (ds_swizzle / ds_bpermute, no memory), is rotated so that the wanted block lines up
// (the bits that wrap around fall on positions the mask discards) and is merged with one bit-select.
template <int S>
__device__ __forceinline__ uint32_t swap_blocks(uint32_t w, uint32_t keep, uint32_t rotate_right)
{
    const uint32_t partner = (uint32_t)__builtin_amdgcn_ds_swizzle((int)w, (S << 10) | 0x1f);    // lane ^ S
    const uint32_t lined_up = __builtin_amdgcn_alignbit(partner, partner, rotate_right);
    return (keep & w) | (~keep & lined_up);
}

__device__ __forceinline__ uint64_t transpose_bits_across_lanes(uint64_t row, int lane)
{
    uint32_t lo = (uint32_t)row, hi = (uint32_t)(row >> 32);
    {   // distance 32: whole words trade places
        const bool lower = (lane & 32) == 0;
        const uint32_t got = (uint32_t)__builtin_amdgcn_ds_bpermute((lane ^ 32) << 2, (int)(lower ? hi : lo));
        const uint32_t nlo = lower ? lo : got, nhi = lower ? got : hi;
        lo = nlo; hi = nhi;
    }
#define MV_SWAP_STAGE(S, MASK)                                                      \
    {                                                                               \
        const bool lower = (lane & S) == 0;                                         \
        const uint32_t keep = lower ? MASK : ~MASK;                                 \
        const uint32_t rot = lower ? 32 - S : S;                                    \
        lo = swap_blocks<S>(lo, keep, rot);                                         \
        hi = swap_blocks<S>(hi, keep, rot);                                         \
    }
    MV_SWAP_STAGE(16, 0x0000ffffu)
    MV_SWAP_STAGE(8, 0x00ff00ffu)
    MV_SWAP_STAGE(4, 0x0f0f0f0fu)
    MV_SWAP_STAGE(2, 0x33333333u)
    MV_SWAP_STAGE(1, 0x55555555u)
#undef MV_SWAP_STAGE
    return ((uint64_t)hi << 32) | lo;
}

// Called by one thread for a world (or a voxel) whose top is `top`: raises the batch's device word and, when
// it rose, the pinned host word (a system-scope atomic maximum, so that two risers cannot leave the smaller
// value behind).
__device__ __forceinline__ void report_height(const HeightFeedback& fb, int top)
{
    if (!fb.device_max) return;
    // thousands of worlds report per upload and almost none of them raises the word: look before the atomic
    if (top <= __hip_atomic_load(fb.device_max, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) return;
    const int old = atomicMax(fb.device_max, top);
    if (top > old) __hip_atomic_fetch_max(fb.host_max, top, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
}

// kPackPrefetch = dwords of the next layer each lane keeps in flight: 8 covers layers up to 2 KiB (40x40), 16
// layers up to 4 KiB (64x64); the deeper variant costs registers, so small layers keep the shallow one.  (Two
// layers in flight per wave change nothing, four are slower: the kernel moves its bytes at the rate of a plain
// device copy as it is.)
// kFastPath = the host has checked that layers are prefetched, 16-byte aligned and one word per row: the other
// paths are then not compiled into the kernel (they cost it a third of its registers, and with them two of its
// eight waves per SIMD).
template <int kPackPrefetch, bool kFastPath>
__global__ __launch_bounds__(kPackThreads) void pack_kernel(const uint8_t* __restrict__ src, uint8_t* __restrict__ vox_dst,
                                                            uint64_t* __restrict__ bits_dst, int32_t* __restrict__ ztop_dst,
                                                            GridLayout g, int vec_ok, const uint8_t* __restrict__ pal_src,
                                                            uint8_t* __restrict__ pal_dst, uint32_t* __restrict__ lut_dst,
                                                            int materials_plus_one, Intensities I, HeightFeedback heights)
{
    extern __shared__ __align__(16) uint8_t layer_lds[];   // one layer per wave, padded to 16 bytes
    __shared__ int top_lds;
    const int env = blockIdx.x;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int waves = kPackThreads / 64;
    const int X = g.X, Y = g.Y, Z = g.Z;
    const int XY = X * Y;
    const int layer_stride = (XY + 15) & ~15;
    uint8_t* mine = layer_lds + (size_t)wave * layer_stride;
    const size_t env_vox = (size_t)env * XY * Z;
    const bool copy = (src != vox_dst);
    uint64_t* xrows = bits_dst + (size_t)env * g.env_words;
    uint64_t* yrows = xrows + g.xrow_words;
    int top = 0;
    const int n4 = XY >> 2;
    const bool prefetch = kFastPath || (vec_ok && n4 <= kPackPrefetch * 64);
    const bool quick = kFastPath || (g.fast && (X & 3) == 0 && XY >= 8 * Y);     // the x rows (8 B each) fit over the layer in LDS
    const bool wide = kFastPath || vec_ok == 2;     // layers and pointers are 16-byte aligned: four dwords per access
    const int n16 = XY >> 4;
    uint32_t pre[kPackPrefetch];
    auto fetch_layer = [&](int k) {
        const uint8_t* layer = src + env_vox + (size_t)k * XY;
        if (wide) {
            const u32x4* s16 = reinterpret_cast<const u32x4*>(layer);
#pragma unroll
            for (int u = 0; u < kPackPrefetch / 4; ++u) {
                u32x4 v = { 0u, 0u, 0u, 0u };
                if (u * 64 + lane < n16) v = __builtin_nontemporal_load(&s16[u * 64 + lane]);
                pre[4 * u] = v.x; pre[4 * u + 1] = v.y; pre[4 * u + 2] = v.z; pre[4 * u + 3] = v.w;
            }
        } else {
            const uint32_t* s4 = reinterpret_cast<const uint32_t*>(layer);
#pragma unroll
            for (int u = 0; u < kPackPrefetch; ++u) pre[u] = (u * 64 + lane) < n4 ? __builtin_nontemporal_load(&s4[u * 64 + lane]) : 0u;
        }
    };
    if (prefetch && wave < Z) fetch_layer(wave);

    // (after the first layers have been requested, so that the palette's trip to memory runs beside theirs)
    if (pal_src) {
        // the environment's palette: private copy, and the colour table lut[face][material]
        const uint8_t* ps = pal_src + (size_t)blockIdx.x * materials_plus_one * 3;
        uint8_t* pd = pal_dst + (size_t)blockIdx.x * materials_plus_one * 3;
        uint32_t* lut = lut_dst + (size_t)blockIdx.x * kNumFaces * materials_plus_one;
        if (ps != pd)
            for (int i = threadIdx.x; i < materials_plus_one * 3; i += kPackThreads) pd[i] = ps[i];
        for (int i = threadIdx.x; i < kNumFaces * materials_plus_one; i += kPackThreads) {
            const int face = i / materials_plus_one, m = i - face * materials_plus_one;
            lut[i] = shade_entry(ps + 3 * m, I.v[face]);
        }
    }
    if (threadIdx.x == 0) top_lds = 0;
    __syncthreads();

    // the rows of layer k from its bytes in this wave's LDS slot
    auto rows_from_lds = [&](int k) {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        uint64_t seen = 0;
        if (quick) {
            // One word per row, X a multiple of 4.  x rows: lane j reads its row as dwords; the non-zero
            // bytes of a dword become a nibble (carry trick + one dot product with weights 1,2,4,8).
            uint32_t lo = 0, hi = 0;
            const uint32_t* rowp = reinterpret_cast<const uint32_t*>(mine + min(lane, Y - 1) * X);
#pragma unroll
            for (int w4 = 0; w4 < 16; ++w4) {
                if (w4 * 4 < X) {
                    const uint32_t x = rowp[w4];
                    const uint32_t flags = ((((x & 0x7f7f7f7fu) + 0x7f7f7f7fu) | x) >> 7) & 0x01010101u;
                    const uint32_t nib = __builtin_amdgcn_udot4(flags, 0x08040201u, 0u, false);
                    if (w4 < 8) lo |= nib << (4 * w4); else hi |= nib << (4 * (w4 - 8));
                }
            }
            const uint64_t xbits = ((uint64_t)hi << 32) | lo;
            seen = xbits;
            if (lane < Y) xrows[(size_t)k * Y + lane] = xbits;
            // y rows = the transpose of the 64x64 bit matrix whose row j is lane j's x row
            const uint64_t ybits = transpose_bits_across_lanes(lane < Y ? xbits : 0ull, lane);
            if (lane < X) yrows[(size_t)k * X + lane] = ybits;
        } else {
            // x rows: row (k*Y + j), word w holds cells i = 64w .. 64w+63
            for (int j0 = 0; j0 < Y; j0 += 64) {
                const int j = min(j0 + lane, Y - 1);
                for (int w = 0; w < g.rowwords_x; ++w) {
                    const uint64_t bits = gather_row_bits(mine + j * X + w * 64, 1, min(64, X - w * 64));
                    seen |= bits;
                    if (j0 + lane < Y) xrows[((size_t)k * Y + j) * g.rowwords_x + w] = bits;
                }
            }
            // y rows: row (k*X + i), word w holds cells j = 64w .. 64w+63
            for (int i0 = 0; i0 < X; i0 += 64) {
                const int i = min(i0 + lane, X - 1);
                for (int w = 0; w < g.rowwords_y; ++w) {
                    const uint64_t bits = gather_row_bits(mine + (w * 64) * X + i, X, min(64, Y - w * 64));
                    if (i0 + lane < X) yrows[((size_t)k * X + i) * g.rowwords_y + w] = bits;
                }
            }
        }
        if (__ballot(seen != 0) != 0) top = k + 1;
        __builtin_amdgcn_wave_barrier();
    };

    if (prefetch) {
        for (int k = wave; k < Z; k += waves) {
            uint8_t* ldst = vox_dst + env_vox + (size_t)k * XY;
            // The private material copy is only ever read at voxels whose occupancy bit is set (the hit
            // voxel of a ray), so a layer without any solid voxel is not copied: its old bytes stay behind
            // bits that are all zero.
            uint32_t any = 0;
#pragma unroll
            for (int u = 0; u < kPackPrefetch; ++u) any |= pre[u];
            const bool solid = __ballot(any != 0) != 0;
            if (!solid && quick) {
                // a layer of air: its rows are zero words, and neither LDS nor the transpose is needed for that
                if (k + waves < Z) fetch_layer(k + waves);
                if (lane < Y) xrows[(size_t)k * Y + lane] = 0ull;
                if (lane < X) yrows[(size_t)k * X + lane] = 0ull;
                continue;
            }
            const bool store_copy = copy && solid;
            if (wide) {
                u32x4* d16 = reinterpret_cast<u32x4*>(ldst);
                u32x4* m16 = reinterpret_cast<u32x4*>(mine);
#pragma unroll
                for (int u = 0; u < kPackPrefetch / 4; ++u) {
                    const int b = u * 64 + lane;
                    if (b < n16) {
                        const u32x4 v = { pre[4 * u], pre[4 * u + 1], pre[4 * u + 2], pre[4 * u + 3] };
                        m16[b] = v;
                        if (store_copy) __builtin_nontemporal_store(v, &d16[b]);
                    }
                }
            } else {
                uint32_t* d4 = reinterpret_cast<uint32_t*>(ldst);
                uint32_t* m4 = reinterpret_cast<uint32_t*>(mine);
#pragma unroll
                for (int u = 0; u < kPackPrefetch; ++u) {
                    const int b = u * 64 + lane;
                    if (b < n4) {
                        m4[b] = pre[u];
                        if (store_copy) __builtin_nontemporal_store(pre[u], &d4[b]);
                    }
                }
            }
            // the next layer is requested as soon as the registers are free, and arrives while this one is packed
            if (k + waves < Z) fetch_layer(k + waves);
            rows_from_lds(k);
        }
    } else {
        for (int k = wave; k < Z; k += waves) {
            const uint8_t* lsrc = src + env_vox + (size_t)k * XY;
            uint8_t* ldst = vox_dst + env_vox + (size_t)k * XY;
            if (vec_ok) {
                const uint32_t* s4 = reinterpret_cast<const uint32_t*>(lsrc);
                uint32_t* d4 = reinterpret_cast<uint32_t*>(ldst);
                uint32_t* m4 = reinterpret_cast<uint32_t*>(mine);
                for (int b = lane; b < n4; b += 64) {
                    uint32_t v = s4[b];
                    m4[b] = v;
                    if (copy) d4[b] = v;
                }
            } else {
                for (int b = lane; b < XY; b += 64) {
                    uint8_t m = lsrc[b];
                    mine[b] = m;
                    if (copy) ldst[b] = m;
                }
            }
            rows_from_lds(k);
        }
    }
    if (lane == 0) atomicMax(&top_lds, top);
    __syncthreads();
    if (threadIdx.x == 0) {
        ztop_dst[env] = top_lds;
        report_height(heights, top_lds);
    }
}

size_t pack_lds_bytes(const GridLayout& g)
{
    const size_t XY = (size_t)g.X * g.Y;
    return ((XY + 15) & ~(size_t)15) * (kPackThreads / 64);
}

hipError_t launch_pack(const uint8_t* src, uint8_t* vox_dst, uint64_t* bits_dst, int32_t* ztop_dst, int count,
                       const GridLayout& g, const uint8_t* pal_src, uint8_t* pal_dst, uint32_t* lut_dst,
                       int materials_plus_one, const float intensity[kNumFaces], const HeightFeedback& heights,
                       hipStream_t stream)
{
    Intensities I;
    for (int f = 0; f < kNumFaces; ++f) I.v[f] = intensity[f];
    const size_t XY = (size_t)g.X * g.Y;
    const size_t lds = pack_lds_bytes(g);
    // 0: byte access; 1: dword access; 2: 16-byte access to the layers (sizes and both pointers aligned)
    int vec_ok = (XY % 4 == 0) && ((reinterpret_cast<uintptr_t>(src) & 3) == 0) &&
                 ((reinterpret_cast<uintptr_t>(vox_dst) & 3) == 0);
    if (vec_ok && XY % 16 == 0 && ((reinterpret_cast<uintptr_t>(src) | reinterpret_cast<uintptr_t>(vox_dst)) & 15) == 0)
        vec_ok = 2;
    const int X = g.X, Y = g.Y;
    const bool quick = g.fast && (X & 3) == 0 && XY >= (size_t)8 * Y;
    const bool deep = XY / 4 > 8 * 64;
    const bool fast_path = vec_ok == 2 && quick && XY / 4 <= (size_t)(deep ? 16 : 8) * 64;
#define MV_LAUNCH_PACK(PREFETCH, FASTPATH)                                                                              \
    hipLaunchKernelGGL((pack_kernel<PREFETCH, FASTPATH>), dim3(count), dim3(kPackThreads), lds, stream, src, vox_dst,    \
                       bits_dst, ztop_dst, g, vec_ok, pal_src, pal_dst, lut_dst, materials_plus_one, I, heights)
    if (!deep) {
        if (fast_path) MV_LAUNCH_PACK(8, true); else MV_LAUNCH_PACK(8, false);
    } else {
        if (fast_path) MV_LAUNCH_PACK(16, true); else MV_LAUNCH_PACK(16, false);
    }
#undef MV_LAUNCH_PACK
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// update: one thread per edited voxel.  The material byte is overwritten; the voxel's bit in its x row
// and in its y row is set or cleared with a 64-bit atomic (several edits of one call may share a row
// word); setting a voxel raises the environment's top-layer bound, clearing never lowers it.
// Two launches per call: kFill == false applies the edits that empty a voxel, kFill == true, after it in
// stream order, those that fill one -- so an object that moves into the voxel another one leaves in the
// same step ends up there whatever the order of the two edits in the list.
// ------------------------------------------------------------------------------------------
template <bool kFill>
__global__ void update_voxels_kernel(const int32_t* __restrict__ env, const int32_t* __restrict__ voxel_index,
                                     const uint8_t* __restrict__ material, int count, uint8_t* __restrict__ vox,
                                     uint64_t* __restrict__ bits, int32_t* __restrict__ ztop, int num_envs,
                                     int voxels_per_env, int num_materials, GridLayout g, HeightFeedback heights)
{
    const int e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= count) return;
    const int n = env[e], idx = voxel_index[e];
    const int m = material ? material[e] : 0;           // no material array: every entry empties its voxel
    if ((m != 0) != kFill) return;
    if (n < 0 || n >= num_envs || idx < 0 || idx >= voxels_per_env || m > num_materials) return;
    const int XY = g.X * g.Y;
    const int k = idx / XY, rem = idx - k * XY, j = rem / g.X, i = rem - j * g.X;
    vox[(size_t)n * voxels_per_env + idx] = (uint8_t)m;
    unsigned long long* xrow = reinterpret_cast<unsigned long long*>(bits) + (size_t)n * g.env_words +
                               ((size_t)k * g.Y + j) * g.rowwords_x + (i >> 6);
    unsigned long long* yrow = reinterpret_cast<unsigned long long*>(bits) + (size_t)n * g.env_words + g.xrow_words +
                               ((size_t)k * g.X + i) * g.rowwords_y + (j >> 6);
    if (kFill) {
        atomicOr(xrow, 1ull << (i & 63));
        atomicOr(yrow, 1ull << (j & 63));
        // (the bound only grows while edits are applied, and hardly any edit raises it: look before the atomic)
        if (__hip_atomic_load(ztop + n, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < k + 1)
            if (atomicMax(ztop + n, k + 1) < k + 1) report_height(heights, k + 1);
    } else {
        atomicAnd(xrow, ~(1ull << (i & 63)));
        atomicAnd(yrow, ~(1ull << (j & 63)));
    }
}

hipError_t launch_update_voxels(const int32_t* env, const int32_t* voxel_index, const uint8_t* material, int count,
                                uint8_t* vox, uint64_t* bits, int32_t* ztop, int num_envs, int voxels_per_env,
                                int num_materials, const GridLayout& g, const HeightFeedback& heights, hipStream_t stream)
{
    hipLaunchKernelGGL(update_voxels_kernel<false>, dim3((count + 255) / 256), dim3(256), 0, stream, env, voxel_index,
                       material, count, vox, bits, ztop, num_envs, voxels_per_env, num_materials, g, heights);
    hipLaunchKernelGGL(update_voxels_kernel<true>, dim3((count + 255) / 256), dim3(256), 0, stream, env, voxel_index,
                       material, count, vox, bits, ztop, num_envs, voxels_per_env, num_materials, g, heights);
    return hipGetLastError();
}

// Objects that moved: every voxel an object left is emptied (first launch, no material array), then every voxel an
// object is in now is filled with the object's material (second launch); negative indices are skipped by the kernel.
hipError_t launch_move_voxels(const int32_t* env, const int32_t* from_voxel, const int32_t* to_voxel,
                              const uint8_t* material, int count, uint8_t* vox, uint64_t* bits, int32_t* ztop,
                              int num_envs, int voxels_per_env, int num_materials, const GridLayout& g,
                              const HeightFeedback& heights, hipStream_t stream)
{
    hipLaunchKernelGGL(update_voxels_kernel<false>, dim3((count + 255) / 256), dim3(256), 0, stream, env, from_voxel,
                       static_cast<const uint8_t*>(nullptr), count, vox, bits, ztop, num_envs, voxels_per_env, num_materials,
                       g, heights);
    hipLaunchKernelGGL(update_voxels_kernel<true>, dim3((count + 255) / 256), dim3(256), 0, stream, env, to_voxel,
                       material, count, vox, bits, ztop, num_envs, voxels_per_env, num_materials, g, heights);
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

constexpr float kBig = 3.0e38f;            // stands in for 1/0: keeps every product finite or +inf, never NaN

__device__ __forceinline__ float safe_rcp(float d)
{
    // v_rcp_f32 (1 ulp) then clamp: +-inf for d = +-0 becomes +-kBig
    return __builtin_amdgcn_fmed3f(__builtin_amdgcn_rcpf(d), -kBig, kBig);
}

// Constants of one scan class of one camera.  A class is (dominant horizontal axis, direction along it,
// direction along the other horizontal axis, vertical direction): class = 8*(y dominant) + 4*(u negative) +
// 2*(v negative) + (z negative), so a ray picks every direction-dependent constant with one record load
// instead of selecting each per ray.  u is the scan axis, v the other horizontal axis.  For negative u
// the class works in mirrored coordinates u' = U - u against a bit-reversed copy of the rows, so that
// inside the traversal every ray runs towards increasing bit positions.  v and z crossings are counted
// without sign; the direction is folded into the address and index steps.
struct alignas(16) ScanClass {
    float Pu;           // camera coordinate along u (mirrored for negative u)
    float uexit;        // U - Pu: distance to the far side of the grid along u
    float dist_v;       // distance from the camera to the first v plane in this direction (>= 0)
    float nv_max;       // v planes between the camera cell and the grid boundary in this direction
    float zero[2];      // 0, 0: where a ray's two crossing counters start (the z counterparts of the two values
                        // above depend on the image row: RowRecord holds them)
    float Pu_err;       // what rounding took from the mirrored coordinate: (U - P) - Pu exactly, 0 if not mirrored
    int   addr0;        // LDS byte address of the camera's row in this class's row array
    int   i0;           // camera cell along u (mirrored)
    int   um1;          // U - 1
    // voxel index of the hit = idx0 + cell*stride_u + n_v*stride_v + n_z*stride_z, evaluated with three fused
    // multiply-adds: every term and partial sum is an integer below 2^24 in magnitude, so float32 is exact
    float idx0;         // voxel index of (mirrored cell 0, camera's v cell, camera's layer)
    float stride_u;     // voxel-index step per mirrored u cell: +-1 (x scans) or +-X (y scans)
    float stride_v;     // voxel-index step per v crossing: +-X (x scans) or +-1 (y scans)
    float stride_z;     // voxel-index step per z crossing: +-X*Y
    int   sv;           // row-address step per v crossing: +-8 bytes
    int   sz;           // row-address step per z crossing: +-8*V bytes
    int   face_u;       // face code of a voxel found while scanning along the row
    int   face_v;       // face code of a voxel entered through a v crossing
    int   face_z;       // face code of a voxel entered through a z crossing
    int   pad;
};
static_assert(sizeof(ScanClass) == 80, "scan class record must be 80 bytes");

// What all pixels of one image row share.  The camera has no roll, so its right axis is horizontal and the vertical
// component of a pixel ray, d_z = F_z + sy*U_z, depends on the row alone: its clamped reciprocal, the parameter of
// the first z crossing and the parameter at which the ray leaves the grid along z are computed once per row when a
// workgroup starts, with the operations a ray would use, instead of once per ray.
struct alignas(16) RowRecord {
    float sy;           // pixel-centre scalar of the row, (H - 2r - 1) / H
    float rcp_z;        // 1 / d_z clamped to +-kBig; its sign is the ray's vertical direction (-0 counts as rising)
    float t0_z;         // parameter of the first z crossing: distance to the first z plane times |1 / d_z|
    float tend_z;       // parameter of the crossing that takes the ray out of the (cut) grid along z
};

// Coarse level (optional): the OR of each pair of neighbouring rows (2J, 2J+1) of a layer, one array per row
// array.  These constants of a scan class sit behind its record, in the same 128-byte slot.
struct alignas(16) PairClass {
    int addr0;          // LDS byte address of the camera's pair row in this class's pair array
    int sv;             // pair-address step when the ray crosses from one pair into the next: +-8 bytes
    int sz;             // pair-address step per z crossing: +-8 * (pairs per layer)
    int inner0;         // 1 if the first v plane ahead of the camera lies inside its pair, 0 if it bounds it
};
static_assert(sizeof(ScanClass) + sizeof(PairClass) <= kClassStride, "class slot too small");

// Plain 3D-DDA through the x rows (any row width), in LDS or in global memory.  Used for grids wider than 64
// voxels, for cameras outside the grid, and for workgroups whose world is taller than the layers staged.  Crossing parameters are t = n*|1/d| + t_first (one fused op, error relative
// to t itself) rather than accumulated.
// self_lo / self_hi: voxels this camera must not see (-1 = none); callers that have already removed the body
// from their copy of the rows pass -1.
__device__ __forceinline__ Hit trace_generic(const uint32_t* __restrict__ xrows32, int rowdwords, const float P[3],
                                             const float d[3], int X, int Y, int Z, bool origin_in_grid, int max_steps,
                                             int self_lo, int self_hi)
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
    if (!origin_in_grid) {
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
    int cell[3], step[3];
    float t_next[3], t_first[3], dt[3], n[3];
    float t_exit = kInf;
#pragma unroll
    for (int a = 0; a < 3; ++a) {
        float q = floorf(fmaf(t0, d[a], P[a]));
        int c = (int)fminf(fmaxf(q, 0.0f), (float)(dim[a] - 1));
        if (a == entry_axis) c = pos[a] ? 0 : dim[a] - 1;
        cell[a] = c;
        step[a] = pos[a] ? 1 : -1;
        float plane = (float)(c + (pos[a] ? 1 : 0));
        t_first[a] = zero[a] ? kInf : (plane - P[a]) * inv[a];
        dt[a] = fabsf(inv[a]);
        n[a] = 0.0f;
        t_next[a] = t_first[a];
        float planes_left = (float)(pos[a] ? dim[a] - 1 - c : c);
        float te = zero[a] ? kInf : fmaf(planes_left, dt[a], t_first[a]);
        t_exit = fminf(t_exit, te);
    }
    auto solid = [&](int i, int j, int k) -> bool {
        const int idx = (k * Y + j) * X + i;
        return ((xrows32[(k * Y + j) * rowdwords + (i >> 5)] >> (i & 31)) & 1u) && idx != self_lo && idx != self_hi;
    };
    int face = entry_axis >= 0 ? 2 * entry_axis + (pos[entry_axis] ? 0 : 1) : 6;
    if (solid(cell[0], cell[1], cell[2])) return Hit{ (cell[2] * Y + cell[1]) * X + cell[0], face, t0 };
    for (int it = 0; it < max_steps; ++it) {
        float tm = fminf(fminf(t_next[0], t_next[1]), t_next[2]);
        if (!(tm < t_exit)) return miss;
        bool cx = (t_next[0] <= t_next[1]) & (t_next[0] <= t_next[2]);
        bool cy = !cx & (t_next[1] <= t_next[2]);
        bool cz = !cx & !cy;
        n[0] += cx ? 1.0f : 0.0f;  cell[0] += cx ? step[0] : 0;
        n[1] += cy ? 1.0f : 0.0f;  cell[1] += cy ? step[1] : 0;
        n[2] += cz ? 1.0f : 0.0f;  cell[2] += cz ? step[2] : 0;
        t_next[0] = fmaf(n[0], dt[0], t_first[0]);
        t_next[1] = fmaf(n[1], dt[1], t_first[1]);
        t_next[2] = fmaf(n[2], dt[2], t_first[2]);
        if (solid(cell[0], cell[1], cell[2])) {
            int axis = cx ? 0 : (cy ? 1 : 2);
            bool p = cx ? pos[0] : (cy ? pos[1] : pos[2]);
            return Hit{ (cell[2] * Y + cell[1]) * X + cell[0], 2 * axis + (p ? 0 : 1), tm };
        }
    }
    return miss;
}

// three-operand forms of the same
__device__ __forceinline__ float vmax3(float a, float b, float c);
__device__ __forceinline__ float vmin3(float a, float b, float c);

// One-instruction min/max: fminf()/fmaxf() make the compiler quiet possible signalling NaNs first
// (an extra v_max per operand inside the loop); no operand here can be one.
__device__ __forceinline__ float vmin(float a, float b)
{
    float r;
    asm("v_min_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
    return r;
}
__device__ __forceinline__ float vmax(float a, float b)
{
    float r;
    asm("v_max_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
    return r;
}
__device__ __forceinline__ float vmax3(float a, float b, float c)
{
    float r;
    asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}
__device__ __forceinline__ float vmin3(float a, float b, float c)
{
    float r;
    asm("v_min3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}

// index of the lowest set bit; the result for 0 is unspecified (callers ignore it for rays that found nothing)
__device__ __forceinline__ int ctz64_nonzero(uint64_t v)
{
    const uint32_t lo = (uint32_t)v, hi = (uint32_t)(v >> 32);
    uint32_t flo, fhi;
    asm("v_ffbl_b32 %0, %1" : "=v"(flo) : "v"(lo));
    asm("v_ffbl_b32 %0, %1" : "=v"(fhi) : "v"(hi));
    // v_ffbl_b32 returns 0xffffffff for 0, so the unsigned minimum picks the low word whenever it has a bit
    return (int)min(flo, 32u + fhi);
}

// v & 1 as a 32-bit operation of its own (the compiler otherwise widens the test back to the 64-bit row)
__device__ __forceinline__ uint32_t low_bit(uint32_t v)
{
    uint32_t b;
    asm("v_and_b32 %0, 1, %1" : "=v"(b) : "v"(v));
    return b;
}

typedef __attribute__((address_space(3))) const uint64_t* lds_u64_ptr;
typedef __attribute__((address_space(3))) const u32x4* lds_u32x4_ptr;

// a*b + c on the 24-bit multiplier (full rate); every product on this path fits 24 x 24 bits.
// mad24s takes the multiplier b from a scalar register (a wave-uniform value such as a grid dimension).
__device__ __forceinline__ int mad24(int a, int b, int c)
{
    int r;
    asm("v_mad_i32_i24 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}
__device__ __forceinline__ int mad24s(int a, int b_uniform, int c)
{
    int r;
    asm("v_mad_i32_i24 %0, %1, %2, %3" : "=v"(r) : "v"(a), "s"(b_uniform), "v"(c));
    return r;
}

// Row-scan traversal: DDA over the (v,z) rows the ray passes through, one 64-bit shift per row.
// The loop has one exit (row holds a solid cell in range, or the ray leaves the grid).  It ends for
// every input: each turn advances n_v or n_z, the crossing parameters n*dt + t0 never decrease, and
// t_end is that same expression at the last plane of each axis, so t_out reaches t_end after at most
// V + Z + 2 turns; a NaN anywhere makes the comparison false and ends it at once.
// n_v and n_z count crossings without sign: the cell is (v0 +- n_v, kc +- n_z), the signs sit in the class.
// kNarrow: both horizontal grid sizes are below 64.  The parameter at which a row is left is capped at
// t_end, which puts the last cell of the run at U at most (U only through rounding at the far boundary);
// with U <= 63 that still is a valid bit position of an always-empty cell, and the clamp to U - 1 that
// 64-cell rows need is left out.
template <bool kNarrow, bool kCoarse>
__device__ __forceinline__ Hit trace_rows(uint32_t classes_addr, float dx, float dy, const RowRecord& rr, int fine_turns)
{
    const bool xm = fabsf(dx) >= fabsf(dy);
    const float du = xm ? dx : dy;
    const float dv = xm ? dy : dx;
    // class = 8*(y dominant) + 4*(u negative) + 2*(v negative) + (z negative): each funnel shift moves the
    // index up one bit and brings in the sign bit of the next component.  Along v and z a component
    // of -0 counts as positive (the ray never crosses a plane of that axis, and the distance to the
    // upper plane is never 0 inside the cell): adding +0 turns -0 into +0 and changes nothing else.
    uint32_t q = xm ? 0u : 1u;
    q = __builtin_amdgcn_alignbit(q, __float_as_uint(du), 31);
    q = __builtin_amdgcn_alignbit(q, __float_as_uint(dv + 0.0f), 31);
    q = __builtin_amdgcn_alignbit(q, __float_as_uint(rr.rcp_z), 31);        // the sign of 1/d_z is the sign of d_z
    const uint32_t qoff = q * (uint32_t)kClassStride;
    ScanClass c;
    {
        lds_u32x4_ptr rec = (lds_u32x4_ptr)(uintptr_t)(classes_addr + qoff);
        u32x4* dst = reinterpret_cast<u32x4*>(&c);
        dst[0] = rec[0]; dst[1] = rec[1]; dst[2] = rec[2]; dst[3] = rec[3]; dst[4] = rec[4];
    }

    const float dua = fabsf(du);
    const float inv_u = safe_rcp(dua);
    const float rcp_v = safe_rcp(dv), rcp_z = rr.rcp_z;
    const float dt_v = fabsf(rcp_v), dt_z = fabsf(rcp_z);
    // first crossing on an axis: the distance to the first plane in the ray's direction times |1/d| (along z: from
    // the image row's record, see RowRecord)
    const float t0_v = c.dist_v * dt_v;
    const float t0_z = rr.t0_z;
    // leaving the grid: same n*dt + t0 expression as the crossings, so the comparison below is exact
    const float t_end = vmin3(c.uexit * inv_u, fmaf(c.nv_max, dt_v, t0_v), rr.tend_z);

    // crossings made so far along v and z (without sign; the directions sit in the class), and the parameters
    // of the next ones: t_v = n_v*dt_v + t0_v, t_z likewise
    // (the counters start from the two zero words of the record: registers the load has filled anyway)
    float t_v, t_z, n_v = c.zero[0], n_z = c.zero[1];
    uint32_t addr = (uint32_t)c.addr0;
    uint64_t r, in_range;
    int i_last;
    // One turn of the loop scans the current row from cell i_from up to the cell i_to where the ray leaves
    // it (parameter t_out = min(t_v, t_z), for narrow grids also capped at t_end): r = row >> i_from,
    // in_range = r << (63 - (i_to - i_from)), non-zero if a solid cell lies in the run; the loop ends there, or
    // when t_out reaches t_end (the ray leaves the grid); otherwise the ray crosses the nearer of the two planes
    // (v first at a tie), the counter of that axis and the row address step, and the crossing parameters are
    // recomputed.  The second shift count is 63 - (i_to - i_from) = (i_from + ~i_to) mod 64: one xor-add, the
    // shifter ignores the upper bits.  Nothing after the loop needs i_from: the hit cell follows from
    // the lowest set bit of in_range and i_to, and bit 0 of r tells whether it is the row's entry cell.
    // The next row is requested as soon as its address is known, at the end of the turn before (render -1 %).
    uint64_t row = 0;
    if constexpr (!kCoarse) row = *(lds_u64_ptr)(uintptr_t)addr;
    int i_a = c.i0, i_b;
    if constexpr (kCoarse) {
        // Coarse level: after `fine_turns` ordinary turns a ray first looks at the PAIR of rows it is in (the OR of
        // rows 2J and 2J+1 of its layer), over the whole run of cells it covers before it leaves the pair or the
        // layer.  An empty run takes it there in one turn (one or two v crossings, or one v crossing and the z
        // crossing, with the very comparisons the ordinary turns would make, so the state it arrives in is the
        // state they would arrive in); otherwise it takes one ordinary turn.  Every decision uses the same
        // crossing parameters as the ordinary scan: the result is the same bit for bit.
        PairClass pc;
        *reinterpret_cast<u32x4*>(&pc) = *(lds_u32x4_ptr)(uintptr_t)(classes_addr + qoff + (uint32_t)sizeof(ScanClass));
        t_v = t0_v; t_z = t0_z;
        uint32_t addr_p = (uint32_t)pc.addr0;
        int inner = pc.inner0;                  // the next v plane lies inside the current pair
        int i_from = i_a;
        r = 0; in_range = 0; i_last = i_from;
        for (int turn = 0;; ++turn) {
            if (turn >= fine_turns) {
                const float t_pair = inner ? fmaf(n_v + 1.0f, dt_v, t0_v) : t_v;     // where the ray leaves the pair along v
                const float t_out = kNarrow ? vmin3(t_pair, t_z, t_end) : vmin(t_pair, t_z);
                const float u_out = fmaf(t_out, dua, c.Pu);
                const int i_to = kNarrow ? (int)u_out : min((int)u_out, c.um1);
                const uint64_t pair_row = *(lds_u64_ptr)(uintptr_t)addr_p;
                const uint64_t pr = pair_row >> i_from;
                const uint64_t pin = pr << ((((i_to) ^ -1) + (i_from)) & 63);
                if (pin == 0) {
                    if (!(t_out < t_end)) { r = pr; in_range = 0; i_last = i_to; break; }   // leaves the grid: a miss
                    if (t_pair <= t_z) {
                        // out of the pair along v: the plane inside it (if it was still ahead) and the one behind it
                        n_v += inner ? 2.0f : 1.0f;
                        addr += (uint32_t)(inner ? 2 * c.sv : c.sv);
                        addr_p += (uint32_t)pc.sv;
                        inner = 1;
                    } else {
                        // the z crossing comes first; the plane inside the pair may still come before it
                        const bool mid = inner && t_v <= t_z;
                        n_v += mid ? 1.0f : 0.0f;
                        addr += (uint32_t)(mid ? c.sv : 0);
                        inner = mid ? 0 : inner;
                        n_z += 1.0f;
                        addr += (uint32_t)c.sz;
                        addr_p += (uint32_t)pc.sz;
                    }
                    t_v = fmaf(n_v, dt_v, t0_v);
                    t_z = fmaf(n_z, dt_z, t0_z);
                    i_from = i_to;
                    continue;
                }
            }
            // an ordinary turn on the row the ray is in
            const uint64_t fine_row = *(lds_u64_ptr)(uintptr_t)addr;
            const float t_out = kNarrow ? vmin3(t_v, t_z, t_end) : vmin(t_v, t_z);
            const float u_out = fmaf(t_out, dua, c.Pu);
            const int i_to = kNarrow ? (int)u_out : min((int)u_out, c.um1);
            r = fine_row >> i_from;
            in_range = r << ((((i_to) ^ -1) + (i_from)) & 63);
            i_last = i_to;
            if ((in_range != 0) | !(t_out < t_end)) break;
            const bool cv = t_v <= t_z;
            if (cv) {
                n_v += 1.0f;
                addr += (uint32_t)c.sv;
                if (!inner) addr_p += (uint32_t)pc.sv;      // that plane bounded the pair
                inner ^= 1;
            } else {
                n_z += 1.0f;
                addr += (uint32_t)c.sz;
                addr_p += (uint32_t)pc.sz;
            }
            t_v = fmaf(n_v, dt_v, t0_v);
            t_z = fmaf(n_z, dt_z, t0_z);
            i_from = i_to;
        }
    } else
    // The loop in assembly: the compiler's structured control flow spends about ten scalar instructions per turn
    // on lane masks (two breaks per trip); written out, a turn needs one, the branch: the two comparisons that
    // decide whether a lane goes on write the execution mask themselves.  Lanes that are done simply leave
    // the execution mask (it only ever shrinks; restored after the loop), so every register of a finished lane
    // keeps the values of its last turn.  The cell index alternates between i_a and i_b from turn to turn; a
    // turn that writes i_a copies it to i_b, so that i_b holds the last cell of a lane whichever turn it left in.
    // The first turn is peeled: it reads the first crossings straight from t0_v / t0_z and starts the crossing
    // counters instead of incrementing them; the loop proper holds four turns per backward branch.  The v-or-z
    // decision of a turn is taken at its top (VCC), well ahead of the selects that read it (a vector instruction may
    // not read a lane mask within two instructions of the one that wrote it).  Every kind of instruction costs this
    // kernel about the same issue time, so what counts is how many there are (measured: the mask-writing
    // comparisons and the longer unrolling together -1.3 %).
    {
        uint64_t exec_save, m_go, m_empty;
        float t_out, tmp;
        int sh;
        // the run of cells [IFROM, ITO] of the current row: ITO from the parameter at which the ray leaves the row
        // (TOUT, NARROW: capped at the grid exit; else the cell is clamped to U - 1), then the two shifts
#define MV_ASM_TEST(TV, TZ, IFROM, ITO, TOUT_AND_CELL, WAIT)                            \
            "v_cmp_le_f32_e32 vcc, " TV ", " TZ "\n\t"                                   \
            TOUT_AND_CELL(TV, TZ, ITO)                                                   \
            WAIT                                                                        \
            "v_lshrrev_b64 %[r], " IFROM ", %[row]\n\t"                                 \
            "v_xad_u32 %[sh], " ITO ", -1, " IFROM "\n\t"                               \
            "v_lshlrev_b64 %[inr], %[sh], %[r]\n\t"
#define MV_ASM_CELL_NARROW(TV, TZ, ITO)                                                 \
            "v_min3_f32 %[tout], " TV ", " TZ ", %[tend]\n\t"                            \
            "v_fma_f32 %[tmp], %[tout], |%[du]|, %[pu]\n\t"                             \
            "v_cvt_i32_f32_e32 " ITO ", %[tmp]\n\t"
#define MV_ASM_CELL_WIDE(TV, TZ, ITO)                                                   \
            "v_min_f32_e32 %[tout], " TV ", " TZ "\n\t"                                  \
            "v_fma_f32 %[tmp], %[tout], |%[du]|, %[pu]\n\t"                             \
            "v_cvt_i32_f32_e32 %[tmp], %[tmp]\n\t"                                      \
            "v_min_i32_e32 " ITO ", %[tmp], %[um1]\n\t"
        // lanes that found a solid cell leave first (their in_range stays non-zero), then the lanes whose ray leaves
        // the grid in this row (theirs is zero): each comparison writes the execution mask itself
#define MV_ASM_LEAVE                                                                    \
            "v_cmpx_eq_u64_e64 %[mempty], 0, %[inr]\n\t"                                \
            "v_cmpx_lt_f32_e64 %[mgo], %[tout], %[tend]\n\t"                            \
            "s_cbranch_execz 2f\n\t"
#define MV_ASM_NEXT_ROW                                                                 \
            "v_cndmask_b32_e32 %[tmp], %[sz], %[sv], vcc\n\t"                           \
            "v_add_u32_e32 %[addr], %[addr], %[tmp]\n\t"                                \
            "ds_read_b64 %[row], %[addr]\n\t"
#define MV_ASM_FIRST_ADVANCE                                                            \
            MV_ASM_NEXT_ROW                                                             \
            "v_cndmask_b32_e64 %[nv], 0, 1.0, vcc\n\t"                                  \
            "v_sub_f32_e32 %[nz], 1.0, %[nv]\n\t"                                       \
            "v_fma_f32 %[tv], %[nv], |%[rv]|, %[t0v]\n\t"                               \
            "v_fma_f32 %[tz], %[nz], |%[rz]|, %[t0z]\n\t"
#define MV_ASM_ADVANCE                                                                  \
            MV_ASM_NEXT_ROW                                                             \
            "v_cndmask_b32_e64 %[tmp], 0, 1.0, vcc\n\t"                                 \
            "v_add_f32_e32 %[nv], %[nv], %[tmp]\n\t"                                    \
            "v_sub_f32_e32 %[tmp], 1.0, %[tmp]\n\t"                                     \
            "v_add_f32_e32 %[nz], %[nz], %[tmp]\n\t"                                    \
            "v_fma_f32 %[tv], %[nv], |%[rv]|, %[t0v]\n\t"                               \
            "v_fma_f32 %[tz], %[nz], |%[rz]|, %[t0z]\n\t"
#define MV_ASM_WAIT "s_waitcnt lgkmcnt(0)\n\t"
#define MV_ASM_TURN_TO_A(CELL)                                                          \
            MV_ASM_TEST("%[tv]", "%[tz]", "%[ib]", "%[ia]", CELL, MV_ASM_WAIT)           \
            "v_mov_b32_e32 %[ib], %[ia]\n\t"                                            \
            MV_ASM_LEAVE                                                                \
            MV_ASM_ADVANCE
#define MV_ASM_TURN_TO_B(CELL)                                                          \
            MV_ASM_TEST("%[tv]", "%[tz]", "%[ia]", "%[ib]", CELL, MV_ASM_WAIT)           \
            MV_ASM_LEAVE                                                                \
            MV_ASM_ADVANCE
        // (the first row has arrived when the statement starts: it is one of its inputs)
#define MV_ASM_LOOP(CELL)                                                               \
            "s_mov_b64 %[save], exec\n\t"                                               \
            MV_ASM_TEST("%[t0v]", "%[t0z]", "%[ia]", "%[ib]", CELL, "")                  \
            MV_ASM_LEAVE                                                                \
            MV_ASM_FIRST_ADVANCE                                                        \
            "1:\n\t"                                                                    \
            MV_ASM_TURN_TO_A(CELL)                                                      \
            MV_ASM_TURN_TO_B(CELL)                                                      \
            MV_ASM_TURN_TO_A(CELL)                                                      \
            MV_ASM_TURN_TO_B(CELL)                                                      \
            "s_branch 1b\n"                                                             \
            "2:\n\t"                                                                    \
            "s_mov_b64 exec, %[save]\n\t"
#define MV_ASM_OPERANDS                                                                                              \
                : [save] "=&s"(exec_save), [mgo] "=&s"(m_go), [mempty] "=&s"(m_empty), [tout] "=&v"(t_out),            \
                  [tmp] "=&v"(tmp), [sh] "=&v"(sh), [r] "=&v"(r), [inr] "=&v"(in_range), [ib] "=&v"(i_b),             \
                  [tv] "=&v"(t_v), [tz] "=&v"(t_z), [ia] "+v"(i_a), [row] "+v"(row), [addr] "+v"(addr),               \
                  [nv] "+v"(n_v), [nz] "+v"(n_z)                                                                      \
                : [tend] "v"(t_end), [du] "v"(du), [pu] "v"(c.Pu), [sv] "v"(c.sv), [sz] "v"(c.sz), [rv] "v"(rcp_v),  \
                  [rz] "v"(rcp_z), [t0v] "v"(t0_v), [t0z] "v"(t0_z), [um1] "v"(c.um1)                                 \
                : "vcc", "scc", "memory"
        if (kNarrow) asm volatile(MV_ASM_LOOP(MV_ASM_CELL_NARROW) MV_ASM_OPERANDS);
        else         asm volatile(MV_ASM_LOOP(MV_ASM_CELL_WIDE) MV_ASM_OPERANDS);
#undef MV_ASM_OPERANDS
#undef MV_ASM_LOOP
#undef MV_ASM_ADVANCE
#undef MV_ASM_FIRST_ADVANCE
#undef MV_ASM_NEXT_ROW
#undef MV_ASM_WAIT
#undef MV_ASM_TURN_TO_A
#undef MV_ASM_TURN_TO_B
#undef MV_ASM_LEAVE
#undef MV_ASM_CELL_WIDE
#undef MV_ASM_CELL_NARROW
#undef MV_ASM_TEST
        i_last = i_b;
    }
    const bool found = in_range != 0;

    // in_range is r moved up so that cell i_last sits at bit 63: its lowest set bit p is cell i_last - (63 - p)
    const int iu = i_last - 63 + ctz64_nonzero(in_range);                        // mirrored cell along u
    const bool along_row = low_bit((uint32_t)r) == 0u;                          // not the row's entry cell
    // the row was entered at the later of the last v crossing and the last z crossing (n-1; for n = 0
    // the expression is <= 0 because the first plane is at most one cell away).  Recomputed with one
    // fused operation each: "t_v - dt_v" would cancel badly for a camera that almost touches a plane.
    const float tv_last = fmaf(n_v - 1.0f, dt_v, t0_v);
    const float tz_last = fmaf(n_z - 1.0f, dt_z, t0_z);
    const bool via_z = tz_last >= tv_last;
    // A hit in the row's entry cell was entered through the later of the two crossings.  The camera's own
    // cell is never solid here (the caller handles that camera before tracing), so the only way to find
    // the entry cell of the first row solid is a camera exactly on a cell boundary looking into the
    // neighbour: both crossings are <= 0 then and the hit is at t = 0 on that boundary.
    const float t_in = vmax3(tv_last, tz_last, 0.0f);
    // distance along u to the near face of the hit cell: the mirrored camera coordinate was rounded once,
    // which matters when the camera almost touches that face; its exact rounding error comes with the class
    const float iu_f = (float)iu;
    const float t_u = ((iu_f - c.Pu) - c.Pu_err) * inv_u;
    const int face_vz = via_z ? c.face_z : c.face_v;
    const int face = along_row ? c.face_u : face_vz;
    const float t = along_row ? t_u : t_in;
    // voxel index: the class record holds the index of (mirrored cell 0, camera's v cell, camera's layer)
    // and the signed index steps per cell along u and per crossing along v and z
    const int idx = (int)fmaf(n_z, c.stride_z, fmaf(n_v, c.stride_v, fmaf(iu_f, c.stride_u, c.idx0)));
    Hit h;
    h.idx = found ? idx : -1;       // face and t are only meaningful for idx >= 0; the caller substitutes the miss values
    h.face = face;
    h.t = t;
    return h;
}

// colour of lane+1 within each group of four lanes (lane 3 of the group keeps its own): DPP
// quad_perm [1,2,3,3]
__device__ __forceinline__ uint32_t next_in_quad(uint32_t v)
{
    // (every lane of a quad is named by the permutation, so no lane falls back on the first operand: with the
    // bound-control bit set the compiler need not initialise one)
    return (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, 0xF9, 0xF, 0xF, true);
}

// COARSE: with the optional second occupancy level (pairs of rows), row-scan grids only
template <bool AUX, bool PACKED, bool FAST, bool COARSE = false>
__global__ __launch_bounds__(1024) __attribute__((amdgpu_waves_per_eu(8, 8))) void render_kernel(RenderParams p)
{
    extern __shared__ __align__(16) uint8_t lds[];
    // A workgroup that has just arrived runs its staging at a raised wave priority (the tile loop returns to the
    // default): its few instructions are issued ahead of the tracing waves it shares the SIMDs with, so its
    // loads are on their way sooner.
    __builtin_amdgcn_s_setprio(3);
    const int threads = p.threads;
    // LDS byte address of the dynamic segment: row addresses in the scan-class records are absolute
    const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t*)lds;

    // XCD-aware mapping: hardware deals workgroup b to XCD b % 8; each XCD gets a contiguous range of
    // observations so that the workgroups sharing an environment also share an L2.  Within the range the
    // workgroups come strip by strip, observation by observation; the last observations are cut into
    // shorter strips (an XCD's work then ends with short workgroups instead of long ones: a shorter tail).
    const uint32_t b = blockIdx.x;
    const uint32_t xcd = b % kXcds, seq = b / kXcds;
    const uint32_t body = (uint32_t)p.obs_body_per_xcd * (uint32_t)p.blocks_per_obs;
    int obs, part, tiles_per_block, strips;
    if (seq < body) {
        obs = (int)(xcd * (uint32_t)p.obs_per_xcd + seq / (uint32_t)p.blocks_per_obs);
        part = (int)(seq % (uint32_t)p.blocks_per_obs);
        tiles_per_block = p.tiles_per_block;
        strips = p.blocks_per_obs;
    } else {
        const uint32_t s2 = seq - body;
        const uint32_t local = (uint32_t)p.obs_body_per_xcd + s2 / (uint32_t)p.blocks_per_obs_tail;
        if (local >= (uint32_t)p.obs_per_xcd) return;
        obs = (int)(xcd * (uint32_t)p.obs_per_xcd + local);
        part = (int)(s2 % (uint32_t)p.blocks_per_obs_tail);
        tiles_per_block = p.tiles_per_block_tail;
        strips = p.blocks_per_obs_tail;
    }
    if (obs >= p.num_obs) return;
    // The hardware deals an XCD's consecutive workgroups to its four shader engines in turn: with an even
    // number of strips per observation the same engines would always get the top strips (mostly sky, the
    // slow ones).  Rotating the strips by a hash of the observation index breaks that pairing.
    if ((strips & 1) == 0) part = (int)(((uint32_t)part + (((uint32_t)obs * 2654435761u) >> 16)) % (uint32_t)strips);
    const int env = obs / p.A;
    if (p.active && p.active[env] == 0) return;         // finished episode: its frame is never drawn
    const GridLayout& g = p.g;
    const int X = g.X, Y = g.Y, Z = g.Z;

    // LDS map, mirrors lds_map() on the host
    const uint32_t off_classes = 0;
    const uint32_t off_scalars = kScanClasses * kClassStride;
    const uint32_t off_rowrec = off_scalars + (uint32_t)((p.W * 4 + 15) & ~15);
    const uint32_t off_lut = off_rowrec + (uint32_t)p.H * 16u;
    const uint32_t off_rows = off_lut + (uint32_t)((kNumFaces * p.materials_plus_one * 4 + 15) & ~15);
    float* lds_sx = reinterpret_cast<float*>(lds + off_scalars);
    RowRecord* lds_rowrec = reinterpret_cast<RowRecord*>(lds + off_rowrec);
    uint64_t* lds_rows = reinterpret_cast<uint64_t*>(lds + off_rows);

    // the camera: uniform for the whole workgroup, read once
    const CameraRecord* __restrict__ recp = p.rec + obs;
    const float P[3] = { recp->P[0], recp->P[1], recp->P[2] };
    const float Fx = recp->F[0], Fy = recp->F[1], Fz = recp->F[2];
    const float Rx = recp->R[0], Ry = recp->R[1], Rz = recp->R[2];
    const float Ux = recp->U[0], Uy = recp->U[1], Uz = recp->U[2];
    const int self_lo = recp->self_lo, self_hi = recp->self_hi;

    const bool origin_in_grid = P[0] >= 0.0f && P[0] <= (float)X && P[1] >= 0.0f && P[1] <= (float)Y &&
                                P[2] >= 0.0f && P[2] <= (float)Z;
    const int k0 = min(max((int)floorf(P[2]), 0), Z - 1);
    // Layers the rays of this camera can reach.  Above the highest solid layer of the environment a rising
    // ray can only miss, so the grid is cut there.  A camera that is itself above every solid sits, for the
    // row scan, in one tall empty layer that reaches from the top of the solids upwards: its layer index is
    // kc = ztop, the plane below it is z = ztop (however far down that is), and only layers 0 .. ztop are
    // ever read (layer ztop is empty by definition).
    const int ztop = p.ztop[env];
    const int kc = min(k0, ztop);
    const int zlim = kc + 1 > ztop ? kc + 1 : ztop;
    // Row scan: only if those layers were staged.  The launch stages as many layers as the tallest world
    // the host has heard of; a taller one is traced through the rows in global memory, cell by cell, and
    // says so, so that the next launch stages enough.
    // Layers kept on chip: the launch reserved LDS for p.staged_layers of them; the batch's device word says how
    // tall the tallest world really is right now (it is exact: written by the pack and edit kernels earlier in the
    // stream), and nothing above that plus the one empty layer on top is worth copying.  A launch whose size was
    // fixed long before it runs (a replayed graph) thus stages only what today's worlds need.
    int staged = FAST ? p.staged_layers : Z;
    if (FAST && p.heights.device_max) {
        const int tallest = __builtin_amdgcn_readfirstlane(__hip_atomic_load(p.heights.device_max, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
        staged = min(staged, max(tallest + 1, 1));
    }
    const bool use_rows = FAST && origin_in_grid && zlim <= staged;
    const int sxw = staged * Y, syw = staged * X;          // words of one staged x / y row array
    if (FAST && origin_in_grid && !use_rows && threadIdx.x == 0 && p.heights.device_max) {
        atomicMax(p.heights.device_max, ztop);
        __hip_atomic_fetch_max(p.heights.host_max, ztop, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
    }

    {   // a3: stage pixel scalars, colour table and this environment's bit rows.
        // The first loads of every stream are issued before any of them is consumed (clamped indices
        // instead of branches keep them in one straight run, and a trip of the row loop fetches four
        // words per thread): the staging then waits for one or two memory round trips instead of five.
        const int tid = threadIdx.x;
        const uint32_t* gl = p.lut + (size_t)env * kNumFaces * p.materials_plus_one;
        uint32_t* ll = reinterpret_cast<uint32_t*>(lds + off_lut);
        const int lut_n = kNumFaces * p.materials_plus_one;
        const float first_sx = p.sx[min(tid, p.W - 1)], first_sy = p.sy[min(tid, p.H - 1)];
        const uint32_t first_lut = gl[min(tid, lut_n - 1)];
        const uint64_t* gb = p.bits + (size_t)env * g.env_words;
        if (FAST) {
            if (use_rows) {
                // arrays: [x rows][x rows mirrored][y rows][y rows mirrored], layers 0 .. staged-1 of each
                uint64_t* ax = lds_rows;
                uint64_t* axm = ax + sxw;
                uint64_t* ay = axm + sxw;
                uint64_t* aym = ay + syw;
                const uint64_t* gy = gb + g.xrow_words;
                const int longest = sxw > syw ? sxw : syw;
                auto row_trip = [&](int base) {
                    const int w0 = base + tid, w1 = w0 + threads;
                    const uint64_t x0 = gb[min(w0, sxw - 1)], x1 = gb[min(w1, sxw - 1)];
                    const uint64_t y0 = gy[min(w0, syw - 1)], y1 = gy[min(w1, syw - 1)];
                    if (w0 < sxw) { ax[w0] = x0; axm[w0] = __brevll(x0) >> (64 - X); }
                    if (w1 < sxw) { ax[w1] = x1; axm[w1] = __brevll(x1) >> (64 - X); }
                    if (w0 < syw) { ay[w0] = y0; aym[w0] = __brevll(y0) >> (64 - Y); }
                    if (w1 < syw) { ay[w1] = y1; aym[w1] = __brevll(y1) >> (64 - Y); }
                };
                row_trip(0);                    // outside the loop: its loads join the three above
                for (int base = 2 * threads; base < longest; base += 2 * threads) row_trip(base);
            }
        } else {
            for (int w = tid; w < g.xrow_words; w += threads) lds_rows[w] = gb[w];
        }
        if (tid < p.W) lds_sx[tid] = first_sx;
        // image row records (see RowRecord); the z constants are those of the two vertical scan directions
        auto row_record = [&](float sy) {
            RowRecord rr;
            rr.sy = sy;
            const float dz = fmaf(sy, Uz, fmaf(first_sx, Rz, Fz));      // R_z = 0: the same for every column
            const bool zneg = (dz + 0.0f) < 0.0f;
            rr.rcp_z = safe_rcp(dz + 0.0f);
            const float dt_z = fabsf(rr.rcp_z);
            // (a rising ray of a camera above the solids leaves the cut grid at its first z plane: any positive
            // distance will do, the top of its real cell is one)
            const float dist_z = fabsf((float)(zneg ? kc : k0 + 1) - P[2]);
            const float nz_max = (float)(zneg ? kc : zlim - 1 - kc);
            rr.t0_z = dist_z * dt_z;
            rr.tend_z = fmaf(nz_max, dt_z, rr.t0_z);
            return rr;
        };
        if (tid < p.H) lds_rowrec[tid] = row_record(first_sy);
        if (tid < lut_n) ll[tid] = first_lut;
        for (int i = tid + threads; i < p.W; i += threads) lds_sx[i] = p.sx[i];
        for (int i = tid + threads; i < p.H; i += threads) lds_rowrec[i] = row_record(p.sy[i]);
        for (int i = tid + threads; i < lut_n; i += threads) ll[i] = gl[i];
    }
    // This workgroup's copy of the rows is private to one camera: the camera's own body is removed from it
    // once, instead of being tested for at every step.  The thread that staged a word (word index modulo the
    // workgroup size) clears the body's bit in it straight after its own stores (one wave's LDS operations
    // keep their order), so the barrier below is the only one the staging needs.
    if (self_lo >= 0) {
#pragma unroll
        for (int part = 0; part < 2; ++part) {
            const int sv_ = part == 0 ? self_lo : self_hi;
            if (sv_ >= 0 && sv_ < X * Y * Z) {
                const int k = sv_ / (X * Y), rem = sv_ - k * X * Y, j = rem / X, i = rem - j * X;
                if (FAST) {
                    if (use_rows && k < staged) {
                        uint64_t* ax = lds_rows;
                        uint64_t* axm = ax + sxw;
                        uint64_t* ay = axm + sxw;
                        uint64_t* aym = ay + syw;
                        if ((int)threadIdx.x == (k * Y + j) % threads) {
                            ax[k * Y + j] &= ~(1ull << i);
                            axm[k * Y + j] &= ~(1ull << (X - 1 - i));
                        }
                        if ((int)threadIdx.x == (k * X + i) % threads) {
                            ay[k * X + i] &= ~(1ull << j);
                            aym[k * X + i] &= ~(1ull << (Y - 1 - j));
                        }
                    }
                } else {
                    const int w = (k * Y + j) * g.rowwords_x + (i >> 6);
                    if ((int)threadIdx.x == w % threads) lds_rows[w] &= ~(1ull << (i & 63));
                }
            }
        }
    }
    // pair arrays (coarse level): [x pairs][x pairs mirrored][y pairs][y pairs mirrored] behind the row arrays
    const int vpx = (Y + 1) / 2, vpy = (X + 1) / 2;         // pairs per layer of the x / y arrays
    const int pxw = staged * vpx, pyw = staged * vpy;
    const uint32_t off_pairs = off_rows + 16u * (uint32_t)(sxw + syw);
    if (use_rows && threadIdx.x >= 64 && threadIdx.x < 64 + kScanClasses) {
        const int q = threadIdx.x - 64;
        const bool xmaj = q < 8, neg = q & 4, vneg = q & 2, zneg = q & 1;
        const int U = xmaj ? X : Y, V = xmaj ? Y : X;
        const float pu = xmaj ? P[0] : P[1], pv = xmaj ? P[1] : P[0];
        ScanClass c;
        c.Pu = neg ? (float)U - pu : pu;
        c.Pu_err = 0.0f;
        c.pad = 0;
        if (neg) {                                         // exact error of the rounded difference (two-sum)
            const float a = (float)U, bneg = -pu;
            const float bb = __fsub_rn(c.Pu, a);
            c.Pu_err = __fadd_rn(__fsub_rn(a, __fsub_rn(c.Pu, bb)), __fsub_rn(bneg, bb));
        }
        c.uexit = (float)U - c.Pu;
        c.i0 = min(max((int)floorf(c.Pu), 0), U - 1);
        // A camera exactly on a u plane belongs to the cell on the + side (cell = floor(P)).  In mirrored
        // coordinates that cell is the one before floor(Pu): start the scan there, so that the neighbour
        // on the - side is found as an ordinary hit along the row (through its u face, at t = 0).
        if (neg && c.Pu == floorf(c.Pu) && c.i0 >= 1 && c.Pu < (float)U) c.i0 -= 1;
        const int j0 = min(max((int)floorf(pv), 0), V - 1);
        // first plane along v: the upper plane of the camera's cell for rising v, the lower one otherwise
        c.dist_v = fabsf((float)(vneg ? j0 : j0 + 1) - pv);
        c.nv_max = (float)(vneg ? j0 : V - 1 - j0);
        c.zero[0] = c.zero[1] = 0.0f;
        const uint32_t array_off = off_rows + 8u * (uint32_t)(xmaj ? (neg ? sxw : 0) : 2 * sxw + (neg ? syw : 0));
        c.addr0 = (int)(lds_base + array_off + 8u * (uint32_t)(kc * V + j0));
        c.sv = vneg ? -8 : 8;
        c.sz = zneg ? -8 * V : 8 * V;
        c.um1 = U - 1;
        c.face_u = 2 * (xmaj ? 0 : 1) + (neg ? 1 : 0);
        c.face_v = 2 * (xmaj ? 1 : 0) + (vneg ? 1 : 0);
        c.face_z = zneg ? 5 : 4;
        const int su = xmaj ? 1 : X;                       // voxel-index step per original u cell
        const int sv_idx = xmaj ? X : 1;                   // and per v cell
        c.stride_u = (float)(neg ? -su : su);
        c.stride_v = (float)(vneg ? -sv_idx : sv_idx);
        c.stride_z = (float)(zneg ? -X * Y : X * Y);
        c.idx0 = (float)(kc * X * Y + j0 * sv_idx + (neg ? (U - 1) * su : 0));
        *reinterpret_cast<ScanClass*>(lds + off_classes + q * kClassStride) = c;
        if (COARSE) {
            const int VP = xmaj ? vpx : vpy;
            PairClass pc;
            const uint32_t pair_off = off_pairs + 8u * (uint32_t)(xmaj ? (neg ? pxw : 0) : 2 * pxw + (neg ? pyw : 0));
            pc.addr0 = (int)(lds_base + pair_off + 8u * (uint32_t)(kc * VP + (j0 >> 1)));
            pc.sv = vneg ? -8 : 8;
            pc.sz = zneg ? -8 * VP : 8 * VP;
            // rising v: the plane above cell j0 lies inside its pair if j0 is even; falling v: the plane below it if j0 is odd
            pc.inner0 = ((j0 & 1) == (vneg ? 1 : 0)) ? 1 : 0;
            *reinterpret_cast<PairClass*>(lds + off_classes + q * kClassStride + sizeof(ScanClass)) = pc;
        }
    }
    __syncthreads();

    if (COARSE && use_rows) {
        const uint64_t* ax = lds_rows;
        const uint64_t* axm = ax + sxw;
        const uint64_t* ay = axm + sxw;
        const uint64_t* aym = ay + syw;
        uint64_t* px = reinterpret_cast<uint64_t*>(lds + off_pairs);
        uint64_t* pxm = px + pxw;
        uint64_t* py = pxm + pxw;
        uint64_t* pym = py + pyw;
        for (int w = threadIdx.x; w < pxw; w += threads) {
            const int k = w / vpx, J = w - k * vpx, a = k * Y + 2 * J;
            const bool two = 2 * J + 1 < Y;
            px[w] = ax[a] | (two ? ax[a + 1] : 0ull);
            pxm[w] = axm[a] | (two ? axm[a + 1] : 0ull);
        }
        for (int w = threadIdx.x; w < pyw; w += threads) {
            const int k = w / vpy, J = w - k * vpy, a = k * X + 2 * J;
            const bool two = 2 * J + 1 < X;
            py[w] = ay[a] | (two ? ay[a + 1] : 0ull);
            pym[w] = aym[a] | (two ? aym[a + 1] : 0ull);
        }
        __syncthreads();
    }

    // A camera inside a solid voxel (its own body is already gone) sees that voxel everywhere, at depth 0
    // with the "inside" face: one test per workgroup instead of one per ray.
    int cam_idx = -1;
    if (use_rows) {
        const int ic = min(max((int)floorf(P[0]), 0), X - 1), jc = min(max((int)floorf(P[1]), 0), Y - 1);
        const uint32_t bit = (uint32_t)(lds_rows[kc * Y + jc] >> ic) & 1u;
        if (__builtin_amdgcn_readfirstlane((int)bit)) cam_idx = (kc * Y + jc) * X + ic;
    }

    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int waves = threads >> 6;
    const int lane = threadIdx.x & 63;
    const int lx = lane % kTileW, ly = lane / kTileW, quad = lane & 3;
    const int lane_pix = ly * p.W + lx;
    const float* sx_lane = lds_sx + lx;
    const RowRecord* rowrec_lane = lds_rowrec + ly;
    const int tile_begin = part * tiles_per_block;
    const int tile_end = min(tile_begin + tiles_per_block, p.tiles_per_obs);
    // per-observation bases: everything inside one observation is addressed with 32-bit offsets
    const size_t obs_pix = (size_t)obs * p.H * p.W;
    float* __restrict__ depth_obs = p.depth + obs_pix;
    uint8_t* __restrict__ rgb_obs = p.rgb + obs_pix * 3;
    uint8_t* __restrict__ auxm_obs = AUX && p.aux_material ? p.aux_material + obs_pix : nullptr;
    int32_t* __restrict__ auxh_obs = AUX && p.aux_hit ? p.aux_hit + obs_pix : nullptr;
    uint8_t* __restrict__ auxf_obs = AUX && p.aux_face ? p.aux_face + obs_pix : nullptr;
    const uint8_t* __restrict__ vox_env = p.vox + (size_t)env * p.voxels_per_env;
    const uint32_t* lut_lds = reinterpret_cast<const uint32_t*>(lds + off_lut);
    const uint32_t last_voxel = (uint32_t)p.voxels_per_env - 1u;
    const int last_material = p.materials_plus_one - 1;

    // a6 + a7 of a finished tile: material -> colour, then the stores.
    // (PACKED launches without auxiliary outputs: `pix` is the wave-uniform pixel offset of the tile, and the two
    // store offsets are a per-lane constant plus a scalar multiple of it)
    const uint32_t lane_depth_off = 4u * (uint32_t)lane_pix, lane_rgb_off = 3u * (uint32_t)lane_pix + (uint32_t)quad;
    auto shade_and_store = [&](int idx, int hit_face, float t, int material, uint32_t pix, bool active, auto trusted_face) {
        // branch-free: lanes that found nothing look up a valid entry as well and then take the miss values
        const bool hit = idx >= 0;
        // (the row scan takes its face codes from the scan-class records: nothing to clamp)
        const int face_row = decltype(trusted_face)::value ? hit_face : min(hit_face, kNumFaces - 1);
        const uint32_t shaded = lut_lds[mad24s(face_row, p.materials_plus_one, min(material, last_material))];
        const uint32_t colour = hit ? shaded : p.sky_packed;
        const float depth = hit ? t : 0.0f;
        const int face = hit ? hit_face : 255;
        material = hit ? material : 0;
        if (PACKED && !AUX) {
            *reinterpret_cast<float*>(reinterpret_cast<uint8_t*>(depth_obs) + (lane_depth_off + 4u * pix)) = depth;
        } else if (active) {
            depth_obs[pix] = depth;
            if (AUX) {
                if (auxm_obs) auxm_obs[pix] = (uint8_t)material;
                if (auxh_obs) auxh_obs[pix] = idx;
                if (auxf_obs) auxf_obs[pix] = (uint8_t)face;
            }
        }
        if (PACKED) {
            // four consecutive lanes hold four consecutive pixels of one row = 12 bytes = three aligned
            // dwords, written by the first three lanes of the quad: dword m holds the upper 4-m bytes'
            // worth of pixel m and the lower m+1 bytes of pixel m+1.
            const uint32_t next = next_in_quad(colour);
            const uint32_t word = (colour >> (8 * quad)) | (next << (24 - 8 * quad));
            if (quad < 3) {
                if (!AUX) *reinterpret_cast<uint32_t*>(rgb_obs + (lane_rgb_off + 3u * pix)) = word;
                else *reinterpret_cast<uint32_t*>(rgb_obs + (3u * pix + (uint32_t)quad)) = word;
            }
        } else if (active) {
            uint8_t* out = rgb_obs + 3u * pix;
            out[0] = (uint8_t)colour;
            out[1] = (uint8_t)(colour >> 8);
            out[2] = (uint8_t)(colour >> 16);
        }
    };

    // The tile loop is software-pipelined by one tile: a trip first requests the material bytes of the tile
    // traced in the previous trip, then traces its own tile, and only then shades and stores the previous
    // one, so that the global fetch hides behind a whole traversal.  (The request is issued in the trip that
    // consumes it: a value still in flight across the loop's back edge would be waited for there.)
    // The loop exists twice: once with the row scan alone (the common case), once with the other tracers,
    // so that the values only those need are not kept in registers through the common loop.
    auto run_tiles = [&](auto rows_only_tag, auto narrow_tag) {
        constexpr bool kRowsOnly = decltype(rows_only_tag)::value;
        constexpr bool kNarrow = decltype(narrow_tag)::value;
        int pend_idx = -1, pend_face = 255;
        float pend_t = 0.0f;
        uint32_t pend_pix = 0;
        bool pend_active = false, pending = false;
        // tile coordinates are carried along instead of divided out of the tile index every trip
        int ty = (tile_begin + wave) / p.tiles_x, tx = (tile_begin + wave) - ty * p.tiles_x - waves;
        for (int tile = tile_begin + wave; tile < tile_end; tile += waves) {
            // lanes without a hit (idx -1 = 0xffffffff) read the last voxel and drop it later: no branch
            const uint8_t pend_material = vox_env[min((uint32_t)pend_idx, last_voxel)];

            tx += waves;
            while (tx >= p.tiles_x) { tx -= p.tiles_x; ++ty; }
            // PACKED launches have W and H multiples of the tile size: every lane owns a pixel, and its
            // addresses are a per-lane constant plus a per-tile (wave-uniform) offset
            bool active = true;
            float sx;
            RowRecord rr;
            uint32_t pix;
            if (PACKED) {
                sx = sx_lane[tx * kTileW];
                rr = rowrec_lane[ty * kTileH];
                pix = AUX ? (uint32_t)(lane_pix + ty * kTileH * p.W + tx * kTileW) : (uint32_t)(ty * kTileH * p.W + tx * kTileW);
            } else {
                const int col = tx * kTileW + lx, row = ty * kTileH + ly;
                active = col < p.W && row < p.H;
                const int ccol = min(col, p.W - 1), crow = min(row, p.H - 1);
                sx = lds_sx[ccol];
                rr = lds_rowrec[crow];
                pix = (uint32_t)mad24s(crow, p.W, ccol);
            }

            // a4: ray through the pixel centre, two fused multiply-adds per axis (the row scan takes what it needs of
            // the vertical component from the row record)
            float d[3];
            d[0] = fmaf(rr.sy, Ux, fmaf(sx, Rx, Fx));
            d[1] = fmaf(rr.sy, Uy, fmaf(sx, Ry, Fy));
            if (!kRowsOnly) d[2] = fmaf(rr.sy, Uz, fmaf(sx, Rz, Fz));

            // a5: traversal
            Hit h;
            if (kRowsOnly) {
                h = trace_rows<kNarrow, COARSE>(lds_base + off_classes, d[0], d[1], rr, p.coarse_after);
            } else if (use_rows) {
                h.idx = cam_idx; h.face = 6; h.t = 0.0f;
            } else if (FAST) {
                // cameras outside the grid, and worlds taller than the staged layers: the x rows in global
                // memory, own body skipped by index
                h = trace_generic(reinterpret_cast<const uint32_t*>(p.bits + (size_t)env * g.env_words), 2 * g.rowwords_x,
                                  P, d, X, Y, Z, origin_in_grid, p.max_steps, self_lo, self_hi);
            } else {
                h = trace_generic(reinterpret_cast<const uint32_t*>(lds_rows), 2 * g.rowwords_x, P, d, X, Y, Z,
                                  origin_in_grid, p.max_steps, -1, -1);
            }

            if (pending) shade_and_store(pend_idx, pend_face, pend_t, pend_material, pend_pix, pend_active, rows_only_tag);
            pend_idx = h.idx; pend_face = h.face; pend_t = h.t;
            pend_pix = pix;
            pend_active = active;
            pending = true;
        }
        if (pending) {
            const uint8_t pend_material = vox_env[min((uint32_t)pend_idx, last_voxel)];
            shade_and_store(pend_idx, pend_face, pend_t, pend_material, pend_pix, pend_active, rows_only_tag);
        }
    };
    __builtin_amdgcn_s_setprio(0);
    if (use_rows && cam_idx < 0) {
        if (X < 64 && Y < 64) run_tiles(std::true_type{}, std::true_type{});
        else run_tiles(std::true_type{}, std::false_type{});
    } else {
        run_tiles(std::false_type{}, std::false_type{});
    }
}

// ------------------------------------------------------------------------------------------
// bars: one workgroup per observation paints the indicator bar over the rendered colours.
// ------------------------------------------------------------------------------------------
__global__ void bars_kernel(uint8_t* __restrict__ rgb, const float* __restrict__ fraction,
                            const uint8_t* __restrict__ active, int A, int W, int H, BarParams bar)
{
    const int obs = blockIdx.x;
    if (active && active[obs / A] == 0) return;
    // number of filled columns: one float32 multiply, one float32 add, floor, clamp
    float cols = floorf(__fadd_rn(__fmul_rn(fraction[obs], (float)bar.width), 0.5f));
    cols = fminf(fmaxf(cols, 0.0f), (float)bar.width);      // NaN falls to 0
    const int filled = (int)cols;
    uint8_t* img = rgb + (size_t)obs * H * W * 3;
    for (int p = threadIdx.x; p < bar.width * bar.height; p += blockDim.x) {
        const int r = p / bar.width, c = p - r * bar.width;
        const uint32_t colour = c < filled ? bar.fill_packed : bar.empty_packed;
        uint8_t* out = img + ((size_t)(bar.y + r) * W + (bar.x + c)) * 3;
        out[0] = (uint8_t)colour;
        out[1] = (uint8_t)(colour >> 8);
        out[2] = (uint8_t)(colour >> 16);
    }
}

hipError_t launch_bars(uint8_t* rgb, const float* fraction, const uint8_t* active, int num_obs, int A, int W, int H,
                       const BarParams& bar, hipStream_t stream)
{
    hipLaunchKernelGGL(bars_kernel, dim3(num_obs), dim3(128), 0, stream, rgb, fraction, active, A, W, H, bar);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// overlay: one workgroup per observation paints the primitives over the rendered colours, one after the
// other; the barrier between two primitives (it also waits for the workgroup's stores) keeps the list order
// where they overlap.
// ------------------------------------------------------------------------------------------
__global__ void overlay_kernel(uint8_t* __restrict__ rgb, const float* __restrict__ values, int values_per_obs,
                               const uint8_t* __restrict__ active, int A, int W, int H, OverlayParams overlay)
{
    const int obs = blockIdx.x;
    if (active && active[obs / A] == 0) return;
    uint8_t* img = rgb + (size_t)obs * H * W * 3;
    for (int k = 0; k < overlay.count; ++k) {
        const OverlayRect& q = overlay.rect[k];
        int filled = 0;
        if (q.kind != 0) {
            // filled columns or rows: one float32 multiply, one float32 add, floor, clamp (NaN falls to 0)
            const int extent = q.kind == 1 ? q.width : q.height;
            float n = floorf(__fadd_rn(__fmul_rn(values[(size_t)obs * values_per_obs + q.value_index], (float)extent), 0.5f));
            n = fminf(fmaxf(n, 0.0f), (float)extent);
            filled = (int)n;
        }
        for (int i = threadIdx.x; i < q.width * q.height; i += blockDim.x) {
            const int r = i / q.width, c = i - r * q.width;
            const bool front = q.kind == 0 || (q.kind == 1 ? c < filled : q.height - 1 - r < filled);
            const uint32_t colour = front ? q.front_packed : q.rest_packed;
            uint8_t* out = img + ((size_t)(q.y + r) * W + (q.x + c)) * 3;
            out[0] = (uint8_t)colour;
            out[1] = (uint8_t)(colour >> 8);
            out[2] = (uint8_t)(colour >> 16);
        }
        if (k + 1 < overlay.count) __syncthreads();
    }
}

hipError_t launch_overlay(uint8_t* rgb, const float* values, int values_per_obs, const uint8_t* active, int num_obs, int A,
                          int W, int H, const OverlayParams& overlay, hipStream_t stream)
{
    hipLaunchKernelGGL(overlay_kernel, dim3(num_obs), dim3(256), 0, stream, rgb, values, values_per_obs, active, A, W, H,
                       overlay);
    return hipGetLastError();
}

__global__ void active_from_done_kernel(const uint8_t* __restrict__ done, uint8_t* __restrict__ active, int n)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) active[i] = done[i] == 0 ? 1 : 0;
}

hipError_t launch_active_from_done(const uint8_t* done, uint8_t* active, int n, hipStream_t stream)
{
    hipLaunchKernelGGL(active_from_done_kernel, dim3((n + 255) / 256), dim3(256), 0, stream, done, active, n);
    return hipGetLastError();
}

template <bool AUX, bool PACKED, bool FAST, bool COARSE = false>
static hipError_t set_lds_limit()
{
    return hipFuncSetAttribute(reinterpret_cast<const void*>(&render_kernel<AUX, PACKED, FAST, COARSE>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsBudget);
}

// Workgroups of the render and pack kernels may ask for more dynamic LDS than the default limit: raise the limit
// of every instantiation to the whole LDS of a compute unit, once per device (the attribute belongs to the
// function on the current device, not to a batch: a value derived from one batch's plan would be wrong for
// the next batch).
hipError_t prepare_kernels()
{
    constexpr int kMaxDevices = 64;
    static std::atomic<bool> done[kMaxDevices];
    int device = 0;
    hipError_t e = hipGetDevice(&device);
    if (e != hipSuccess) return e;
    if (device >= 0 && device < kMaxDevices && done[device].load(std::memory_order_acquire)) return hipSuccess;
#define MV_SET(A, P, F) if (e == hipSuccess) e = set_lds_limit<A, P, F>()
    MV_SET(false, false, false); MV_SET(false, false, true); MV_SET(false, true, false); MV_SET(false, true, true);
    MV_SET(true, false, false);  MV_SET(true, false, true);  MV_SET(true, true, false);  MV_SET(true, true, true);
#undef MV_SET
#define MV_SET(A, P) if (e == hipSuccess) e = set_lds_limit<A, P, true, true>()
    MV_SET(false, false); MV_SET(false, true); MV_SET(true, false); MV_SET(true, true);
#undef MV_SET
    // the pack kernel also has a few static words of LDS: its dynamic share must leave room for them
    const int pack_limit = (int)(kLdsBudget - kPackStaticLds);
#define MV_SET(N, F)                                                                                              \
    if (e == hipSuccess)                                                                                          \
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(&pack_kernel<N, F>),                                \
                                hipFuncAttributeMaxDynamicSharedMemorySize, pack_limit)
    MV_SET(8, false); MV_SET(8, true); MV_SET(16, false); MV_SET(16, true);
#undef MV_SET
    if (e == hipSuccess && device >= 0 && device < kMaxDevices) done[device].store(true, std::memory_order_release);
    return e;
}

hipError_t launch_render(const RenderParams& p, size_t lds_bytes, hipStream_t stream)
{
    const bool aux = p.aux_material || p.aux_hit || p.aux_face;
    // dword colour stores and unclamped tiles need whole 8x8 tiles and a 4-byte aligned colour tensor
    const bool packed = (p.W % kTileW == 0) && (p.H % kTileH == 0) && ((reinterpret_cast<uintptr_t>(p.rgb) & 3) == 0);
    const bool fast = p.g.fast != 0;
    dim3 grid(p.blocks_per_xcd * kXcds), block(p.threads);
#define MV_LAUNCH(A, P, F) hipLaunchKernelGGL((render_kernel<A, P, F>), grid, block, lds_bytes, stream, p)
#define MV_LAUNCH_COARSE(A, P) hipLaunchKernelGGL((render_kernel<A, P, true, true>), grid, block, lds_bytes, stream, p)
    if (fast && p.coarse_after >= 0) {
        if (aux) { if (packed) MV_LAUNCH_COARSE(true, true); else MV_LAUNCH_COARSE(true, false); }
        else     { if (packed) MV_LAUNCH_COARSE(false, true); else MV_LAUNCH_COARSE(false, false); }
    } else if (aux) {
        if (packed) { if (fast) MV_LAUNCH(true, true, true); else MV_LAUNCH(true, true, false); }
        else        { if (fast) MV_LAUNCH(true, false, true); else MV_LAUNCH(true, false, false); }
    } else {
        if (packed) { if (fast) MV_LAUNCH(false, true, true); else MV_LAUNCH(false, true, false); }
        else        { if (fast) MV_LAUNCH(false, false, true); else MV_LAUNCH(false, false, false); }
    }
#undef MV_LAUNCH_COARSE
#undef MV_LAUNCH
    return hipGetLastError();
}

}  // namespace mv
