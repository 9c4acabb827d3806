// Issue rate of single vector instructions on gfx950: a measurement tool, not part of the library.
//
// The render kernel is bound by vector-ALU issue, so its roofline needs to know what one vector
// instruction costs.  Each probe runs one instruction kind in eight independent register chains, 16
// instructions per loop trip, on 8 waves per SIMD of every CU (2048 workgroups of 256 threads), and
// reports cycles per wave-instruction per SIMD at the nominal 2.4 GHz.  The loops touch no memory;
// every kernel ends after `iters` trips.  A last probe reads the shader clock against the 100 MHz
// wall clock while the vector ALUs are busy.
//
// Build: hipcc -O3 --offload-arch=gfx950 -o valu_rates valu_rates.hip      Run: ./valu_rates
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>

#define CK(x)                                                                                   \
    do {                                                                                        \
        hipError_t e_ = (x);                                                                    \
        if (e_ != hipSuccess) {                                                                 \
            std::printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__);          \
            return 1;                                                                           \
        }                                                                                       \
    } while (0)

// chains: f0..f7 float, u0..u7 dword, q0..q7 qword; s0..s7 receive compare masks
#define CHAINS                                                                                  \
    const int l = threadIdx.x & 63;                                                             \
    float f0 = l, f1 = l + 1, f2 = l + 2, f3 = l + 3, f4 = l + 4, f5 = l + 5, f6 = l + 6, f7 = l + 7; \
    uint32_t u0 = l, u1 = l + 1, u2 = l + 2, u3 = l + 3, u4 = l + 4, u5 = l + 5, u6 = l + 6, u7 = l + 7; \
    uint64_t q0 = l, q1 = l + 1, q2 = l + 2, q3 = l + 3, q4 = l + 4, q5 = l + 5, q6 = l + 6, q7 = l + 7; \
    uint64_t s0 = 0, s1 = 0, s2 = 0, s3 = 0, s4 = 0, s5 = 0, s6 = 0, s7 = 0;                    \
    const float fb = 1.0001f + l * 1e-6f, fc = 0.5f;                                            \
    const uint32_t ub = 0x9e3779b9u * (l + 1), uc = (l & 7) + 1;                                \
    const uint64_t smask = 0x5555aaaa5555aaaaull;                                               \
    (void)fc; (void)ub; (void)uc; (void)smask;
#define RESULT                                                                                  \
    out[blockIdx.x * blockDim.x + threadIdx.x] = f0 + f1 + f2 + f3 + f4 + f5 + f6 + f7 +        \
        (float)(u0 ^ u1 ^ u2 ^ u3 ^ u4 ^ u5 ^ u6 ^ u7) + (float)(q0 ^ q1 ^ q2 ^ q3 ^ q4 ^ q5 ^ q6 ^ q7) + \
        (float)(s0 ^ s1 ^ s2 ^ s3 ^ s4 ^ s5 ^ s6 ^ s7);
#define EIGHT(S) S(0) S(1) S(2) S(3) S(4) S(5) S(6) S(7)
#define PROBE(NAME, S)                                                                          \
    __global__ __launch_bounds__(256) void NAME(float* out, int iters)                          \
    {                                                                                           \
        CHAINS                                                                                  \
        for (int it = 0; it < iters; ++it) { EIGHT(S) EIGHT(S) }                                \
        RESULT                                                                                  \
    }

// full-rate candidates
#define S_FMA(i)     asm volatile("v_fma_f32 %0, %0, %1, %2" : "+v"(f##i) : "v"(fb), "v"(fc));
#define S_ADDF(i)    asm volatile("v_add_f32 %0, %0, %1" : "+v"(f##i) : "v"(fb));
#define S_MULF(i)    asm volatile("v_mul_f32 %0, %0, %1" : "+v"(f##i) : "v"(fb));
#define S_MOV(i)     asm volatile("v_mov_b32 %0, %1" : "=v"(u##i) : "v"(ub));
#define S_AND(i)     asm volatile("v_and_b32 %0, %0, %1" : "+v"(u##i) : "v"(ub));
#define S_ADDU(i)    asm volatile("v_add_u32 %0, %0, %1" : "+v"(u##i) : "v"(ub));
#define S_LSHR(i)    asm volatile("v_lshrrev_b32 %0, %1, %0" : "+v"(u##i) : "v"(uc));
#define S_ASHR(i)    asm volatile("v_ashrrev_i32 %0, 31, %0" : "+v"(u##i));
// the rest of what the render kernel's traversal uses
#define S_MINF(i)    asm volatile("v_min_f32 %0, %0, %1" : "+v"(f##i) : "v"(fb));
#define S_MIN3F(i)   asm volatile("v_min3_f32 %0, %0, %1, %2" : "+v"(f##i) : "v"(fb), "v"(fc));
#define S_MED3F(i)   asm volatile("v_med3_f32 %0, %0, %1, %2" : "+v"(f##i) : "v"(fb), "v"(fc));
#define S_CMPF(i)    asm volatile("v_cmp_lt_f32 %0, %1, %2" : "=s"(s##i) : "v"(f##i), "v"(fb));
#define S_CMPQ(i)    asm volatile("v_cmp_eq_u64 %0, 0, %1" : "=s"(s##i) : "v"(q##i));
#define S_CNDMASK(i) asm volatile("v_cndmask_b32 %0, %0, %1, %2" : "+v"(u##i) : "v"(ub), "s"(smask));
#define S_CVTIF(i)   asm volatile("v_cvt_i32_f32 %0, %1" : "=v"(u##i) : "v"(f##i));
#define S_CVTFI(i)   asm volatile("v_cvt_f32_i32 %0, %1" : "=v"(f##i) : "v"(u##i));
#define S_MINI(i)    asm volatile("v_min_i32 %0, %0, %1" : "+v"(u##i) : "v"(ub));
#define S_LSHL(i)    asm volatile("v_lshlrev_b32 %0, %1, %0" : "+v"(u##i) : "v"(uc));
#define S_LSHRQ(i)   asm volatile("v_lshrrev_b64 %0, %1, %0" : "+v"(q##i) : "v"(uc));
#define S_LSHLQ(i)   asm volatile("v_lshlrev_b64 %0, %1, %0" : "+v"(q##i) : "v"(uc));
#define S_XAD(i)     asm volatile("v_xad_u32 %0, %0, %1, %2" : "+v"(u##i) : "v"(uc), "v"(ub));
#define S_ADD3(i)    asm volatile("v_add3_u32 %0, %0, %1, %2" : "+v"(u##i) : "v"(ub), "v"(uc));
#define S_MAD24(i)   asm volatile("v_mad_i32_i24 %0, %0, %1, %2" : "+v"(u##i) : "v"(ub), "v"(uc));
#define S_FFBL(i)    asm volatile("v_ffbl_b32 %0, %0" : "+v"(u##i));
#define S_DPP(i)     asm volatile("v_mov_b32_dpp %0, %1 quad_perm:[1,2,3,3] row_mask:0xf bank_mask:0xf" : "+v"(u##i) : "v"(ub));
#define S_RCP(i)     asm volatile("v_rcp_f32 %0, %0" : "+v"(f##i));

PROBE(k_fma, S_FMA) PROBE(k_addf, S_ADDF) PROBE(k_mulf, S_MULF) PROBE(k_mov, S_MOV) PROBE(k_and, S_AND)
PROBE(k_addu, S_ADDU) PROBE(k_lshr, S_LSHR) PROBE(k_ashr, S_ASHR)
PROBE(k_minf, S_MINF) PROBE(k_min3f, S_MIN3F) PROBE(k_med3f, S_MED3F) PROBE(k_cmpf, S_CMPF) PROBE(k_cmpq, S_CMPQ)
PROBE(k_cndmask, S_CNDMASK) PROBE(k_cvtif, S_CVTIF) PROBE(k_cvtfi, S_CVTFI) PROBE(k_mini, S_MINI)
PROBE(k_lshl, S_LSHL) PROBE(k_lshrq, S_LSHRQ) PROBE(k_lshlq, S_LSHLQ) PROBE(k_xad, S_XAD) PROBE(k_add3, S_ADD3)
PROBE(k_mad24, S_MAD24) PROBE(k_ffbl, S_FFBL) PROBE(k_dpp, S_DPP) PROBE(k_rcp, S_RCP)

// shader clock against the 100 MHz wall clock under a full vector load
__global__ __launch_bounds__(256) void k_clock(float* out, unsigned long long* ticks, int iters)
{
    CHAINS
    const unsigned long long c0 = clock64(), w0 = wall_clock64();
    for (int it = 0; it < iters; ++it) { EIGHT(S_FMA) EIGHT(S_FMA) }
    const unsigned long long c1 = clock64(), w1 = wall_clock64();
    if (blockIdx.x == 0 && threadIdx.x == 0) { ticks[0] = c1 - c0; ticks[1] = w1 - w0; }
    RESULT
}

typedef void (*probe_fn)(float*, int);
struct Probe { const char* name; probe_fn fn; };

int main()
{
    const int blocks = 256 * 8, threads = 256, iters = 4000;
    const Probe probes[] = {
        {"v_fma_f32", k_fma}, {"v_add_f32", k_addf}, {"v_mul_f32", k_mulf}, {"v_mov_b32", k_mov}, {"v_and_b32", k_and},
        {"v_add_u32", k_addu}, {"v_lshrrev_b32", k_lshr}, {"v_ashrrev_i32", k_ashr},
        {"v_min_f32", k_minf}, {"v_min3_f32", k_min3f}, {"v_med3_f32", k_med3f}, {"v_cmp_lt_f32", k_cmpf},
        {"v_cmp_eq_u64", k_cmpq}, {"v_cndmask_b32", k_cndmask}, {"v_cvt_i32_f32", k_cvtif}, {"v_cvt_f32_i32", k_cvtfi},
        {"v_min_i32", k_mini}, {"v_lshlrev_b32", k_lshl}, {"v_lshrrev_b64", k_lshrq}, {"v_lshlrev_b64", k_lshlq},
        {"v_xad_u32", k_xad}, {"v_add3_u32", k_add3}, {"v_mad_i32_i24", k_mad24}, {"v_ffbl_b32", k_ffbl},
        {"v_mov_b32 (dpp)", k_dpp}, {"v_rcp_f32", k_rcp},
    };
    float* out = nullptr;
    unsigned long long* ticks = nullptr;
    CK(hipMalloc(&out, sizeof(float) * blocks * threads));
    CK(hipMalloc(&ticks, 2 * sizeof(unsigned long long)));
    hipEvent_t e0, e1;
    CK(hipEventCreate(&e0));
    CK(hipEventCreate(&e1));

    hipLaunchKernelGGL(k_fma, dim3(blocks), dim3(threads), 0, 0, out, 10 * iters);        // warm the clocks up
    CK(hipDeviceSynchronize());
    for (int rep = 0; rep < 3; ++rep) {
        unsigned long long h[2];
        hipLaunchKernelGGL(k_clock, dim3(blocks), dim3(threads), 0, 0, out, ticks, 10 * iters);
        CK(hipDeviceSynchronize());
        CK(hipMemcpy(h, ticks, sizeof(h), hipMemcpyDeviceToHost));
        std::printf("shader clock under v_fma_f32 load: %.0f MHz\n", (double)h[0] / ((double)h[1] / 100.0));
    }
    const double wave_insts_per_simd = (double)blocks * (threads / 64) * iters * 16 / 1024.0;
    std::printf("%-18s %10s %28s\n", "instruction", "ms", "cycles per wave-instruction");
    for (const Probe& p : probes) {
        hipLaunchKernelGGL(p.fn, dim3(blocks), dim3(threads), 0, 0, out, iters);
        CK(hipDeviceSynchronize());
        CK(hipEventRecord(e0, 0));
        hipLaunchKernelGGL(p.fn, dim3(blocks), dim3(threads), 0, 0, out, iters);
        CK(hipEventRecord(e1, 0));
        CK(hipEventSynchronize(e1));
        float ms = 0.0f;
        CK(hipEventElapsedTime(&ms, e0, e1));
        std::printf("%-18s %10.3f %28.2f\n", p.name, ms, ms * 1e-3 * 2.4e9 / wave_insts_per_simd);
        std::fflush(stdout);
    }
    CK(hipEventDestroy(e0));
    CK(hipEventDestroy(e1));
    CK(hipFree(ticks));
    CK(hipFree(out));
    return 0;
}
