// Measurement aid, not a layer and not part of libsmall_hip: a register-resident loop of independent fp32 matrix
// instructions, to read the matrix rate this chip actually sustains (the benchmark quotes roofline fractions against
// the published peak and against this). Built into a library of its own (libsmall_probe.so, include/small_probe.h).
// Every wave runs `iters` rounds of eight independent v_mfma_f32_16x16x4_f32 accumulations on operands it never
// reloads and stores one value at the end so that nothing is optimised away.
#include "../../include/small_probe.h"

#include <hip/hip_runtime.h>

namespace {

typedef float floatx4 __attribute__((ext_vector_type(4)));

__global__ void __launch_bounds__(256) mfma_probe_kernel(float *out, int iters, float seed)
{
    floatx4 acc[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) acc[k] = floatx4{0.f, 0.f, 0.f, 0.f};
    const float a = seed + (float)(threadIdx.x & 7) * 1e-3f, b = 1.0f - seed;
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int k = 0; k < 8; ++k) acc[k] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, acc[k], 0, 0, 0);
    }
    float sum = 0.f;
#pragma unroll
    for (int k = 0; k < 8; ++k) sum += acc[k][0] + acc[k][1] + acc[k][2] + acc[k][3];
    out[(size_t)blockIdx.x * 256 + threadIdx.x] = sum;
}

// The same loop with vector-ALU work beside it: per round sixteen matrix instructions (four accumulators, four
// steps each) and VALU independent fp32 multiply-adds on eight registers of their own, the multiply-adds first.
// Written as one block of instructions per round so that the compiler neither reorders nor removes any: what the
// round costs beyond its matrix instructions is what a vector instruction costs next to the matrix pipe.
#define SMALL_FM8 \
    "v_fmac_f32 %[f0], %[a], %[b]\n\tv_fmac_f32 %[f1], %[a], %[b]\n\tv_fmac_f32 %[f2], %[a], %[b]\n\tv_fmac_f32 %[f3], %[a], %[b]\n\t" \
    "v_fmac_f32 %[f4], %[a], %[b]\n\tv_fmac_f32 %[f5], %[a], %[b]\n\tv_fmac_f32 %[f6], %[a], %[b]\n\tv_fmac_f32 %[f7], %[a], %[b]\n\t"
#define SMALL_MF4 \
    "v_mfma_f32_16x16x4_f32 %[c0], %[a], %[b], %[c0]\n\tv_mfma_f32_16x16x4_f32 %[c1], %[a], %[b], %[c1]\n\t" \
    "v_mfma_f32_16x16x4_f32 %[c2], %[a], %[b], %[c2]\n\tv_mfma_f32_16x16x4_f32 %[c3], %[a], %[b], %[c3]\n\t"
#define SMALL_FM16 SMALL_FM8 SMALL_FM8
#define SMALL_FM32 SMALL_FM16 SMALL_FM16
#define SMALL_MIX_KERNEL(NAME, VALU_TEXT)                                                                                 \
    __global__ void __launch_bounds__(256) NAME(float *out, int iters, float seed)                                        \
    {                                                                                                                     \
        floatx4 c0 = {0.f, 0.f, 0.f, 0.f}, c1 = c0, c2 = c0, c3 = c0;                                                     \
        float f0 = 0.f, f1 = 0.f, f2 = 0.f, f3 = 0.f, f4 = 0.f, f5 = 0.f, f6 = 0.f, f7 = 0.f;                             \
        const float a = seed + (float)(threadIdx.x & 7) * 1e-3f, b = 1.0f - seed;                                         \
        for (int i = 0; i < iters; ++i)                                                                                   \
            asm volatile(VALU_TEXT SMALL_MF4 SMALL_MF4 SMALL_MF4 SMALL_MF4                                                \
                         : [c0] "+v"(c0), [c1] "+v"(c1), [c2] "+v"(c2), [c3] "+v"(c3), [f0] "+v"(f0), [f1] "+v"(f1),      \
                           [f2] "+v"(f2), [f3] "+v"(f3), [f4] "+v"(f4), [f5] "+v"(f5), [f6] "+v"(f6), [f7] "+v"(f7)       \
                         : [a] "v"(a), [b] "v"(b));                                                                       \
        const floatx4 c = c0 + c1 + c2 + c3;                                                                              \
        out[(size_t)blockIdx.x * 256 + threadIdx.x] = c[0] + c[1] + c[2] + c[3] + (f0 + f1 + f2 + f3 + f4 + f5 + f6 + f7); \
    }
SMALL_MIX_KERNEL(mix_probe_0, "")
SMALL_MIX_KERNEL(mix_probe_32, SMALL_FM32)
SMALL_MIX_KERNEL(mix_probe_64, SMALL_FM32 SMALL_FM32)
SMALL_MIX_KERNEL(mix_probe_96, SMALL_FM32 SMALL_FM32 SMALL_FM32)

}  // namespace

extern "C" int small_probe_mfma_valu(float *out, int workgroups, int iters, int valu, void *stream)
{
    if (!out) return 1;
    if (workgroups <= 0 || workgroups > (1 << 20) || iters <= 0) return 2;
    if (valu != 0 && valu != 32 && valu != 64 && valu != 96) return 2;
    const hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    const dim3 grid((unsigned)workgroups), block(256);
    if (valu == 0) hipLaunchKernelGGL(mix_probe_0, grid, block, 0, s, out, iters, 0.25f);
    else if (valu == 32) hipLaunchKernelGGL(mix_probe_32, grid, block, 0, s, out, iters, 0.25f);
    else if (valu == 64) hipLaunchKernelGGL(mix_probe_64, grid, block, 0, s, out, iters, 0.25f);
    else hipLaunchKernelGGL(mix_probe_96, grid, block, 0, s, out, iters, 0.25f);
    return hipGetLastError() == hipSuccess ? 0 : 5;
}

extern "C" int small_probe_mfma(float *out, int workgroups, int iters, void *stream)
{
    if (!out) return 1;
    if (workgroups <= 0 || workgroups > (1 << 20) || iters <= 0) return 2;
    hipLaunchKernelGGL(mfma_probe_kernel, dim3((unsigned)workgroups), dim3(256), 0, reinterpret_cast<hipStream_t>(stream), out,
                       iters, 0.25f);
    return hipGetLastError() == hipSuccess ? 0 : 5;
}
