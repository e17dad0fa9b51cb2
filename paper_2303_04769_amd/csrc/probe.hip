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

}  // namespace

extern "C" int small_probe_mfma(float *out, int workgroups, int iters, void *stream)
{
    if (!out) return 1;
    if (workgroups <= 0 || workgroups > (1 << 20) || iters <= 0) return 2;
    hipLaunchKernelGGL(mfma_probe_kernel, dim3((unsigned)workgroups), dim3(256), 0, reinterpret_cast<hipStream_t>(stream), out,
                       iters, 0.25f);
    return hipGetLastError() == hipSuccess ? 0 : 5;
}
