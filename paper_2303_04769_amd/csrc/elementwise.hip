// Single-element reductions (paper Table 1 row 1: ReLU, addition) and the layout
// conversions of Section 4.4 "Common Data Format". All HBM-bound: 16-byte accesses,
// consecutive lanes on consecutive addresses, no matrix cores.
#include "small_internal.h"

namespace small {

namespace {

constexpr int kBlock = 256;
constexpr int kVecPerThread = 1;   // float4 items per thread (1 measured fastest for streaming on MI355X)

__device__ __forceinline__ float relu1(float x) { return (x > 0.0f) ? x : 0.0f; }

// One block covers kBlock * kVecPerThread consecutive float4 items. `out` may equal an input
// exactly (in place): each thread reads all of its items before it writes any of them.
template <bool kAdd>
__global__ void __launch_bounds__(kBlock) ew_vec4(const floatx4 *a, const floatx4 *b, floatx4 *out, size_t n4)
{
    const size_t base = (size_t)blockIdx.x * (kBlock * kVecPerThread) + threadIdx.x;
    floatx4 va[kVecPerThread], vb[kVecPerThread];
#pragma unroll
    for (int i = 0; i < kVecPerThread; ++i) {
        const size_t k = base + (size_t)i * kBlock;
        if (k < n4) {
            va[i] = __builtin_nontemporal_load(a + k);
            if (kAdd) vb[i] = __builtin_nontemporal_load(b + k);
        }
    }
#pragma unroll
    for (int i = 0; i < kVecPerThread; ++i) {
        const size_t k = base + (size_t)i * kBlock;
        if (k < n4) {
            floatx4 r;
            if (kAdd) {
                r = va[i] + vb[i];
            } else {
                r.x = relu1(va[i].x); r.y = relu1(va[i].y); r.z = relu1(va[i].z); r.w = relu1(va[i].w);
            }
            __builtin_nontemporal_store(r, out + k);
        }
    }
}

template <bool kAdd>
__global__ void __launch_bounds__(kBlock) ew_scalar(const float *a, const float *b, float *out, size_t begin, size_t n)
{
    const size_t k = begin + (size_t)blockIdx.x * kBlock + threadIdx.x;
    if (k < n) out[k] = kAdd ? (a[k] + b[k]) : relu1(a[k]);
}

template <bool kAdd>
hipError_t launch_ew(const float *a, const float *b, float *out, size_t n, hipStream_t s)
{
    if (n == 0) return hipSuccess;
    const bool aligned = (((uintptr_t)a | (uintptr_t)out | (kAdd ? (uintptr_t)b : 0)) & 15u) == 0;
    size_t n4 = aligned ? n / 4 : 0;
    if (n4) {
        const size_t per_block = (size_t)kBlock * kVecPerThread;
        const size_t blocks = (n4 + per_block - 1) / per_block;
        hipLaunchKernelGGL(ew_vec4<kAdd>, dim3((unsigned)blocks), dim3(kBlock), 0, s, (const floatx4 *)a,
                           (const floatx4 *)b, (floatx4 *)out, n4);
    }
    const size_t done = n4 * 4;
    if (done < n) {
        const size_t blocks = (n - done + kBlock - 1) / kBlock;
        hipLaunchKernelGGL(ew_scalar<kAdd>, dim3((unsigned)blocks), dim3(kBlock), 0, s, a, b, out, done, n);
    }
    return hipGetLastError();
}

// ---- plain <-> blocked activations.
// One block moves a tile of Cb channels x kPix pixels of one (image, channel block) through
// LDS, so both the plain side (contiguous along H*W) and the blocked side (contiguous
// along [pixel][Cb]) see coalesced accesses. Pure copy: bit-exact.
constexpr int kPix = 64;

template <bool kUnpack>
__global__ void __launch_bounds__(kBlock) pack_tile(float *__restrict__ plain_base, float *__restrict__ blk_base,
                                                     int C, int HW, int Cb)
{
    __shared__ float tile[64][kPix + 1];   // [channel in block][pixel], Cb <= 64
    const int nCb = C / Cb;
    const int plane = blockIdx.x;          // n * nCb + cb
    const int n = plane / nCb, cb = plane - n * nCb;
    const int p0 = blockIdx.y * kPix;
    const int np = min(kPix, HW - p0);
    float *plain = plain_base + ((size_t)n * C + (size_t)cb * Cb) * HW + p0;   // Cb rows of HW floats
    float *blk = blk_base + ((size_t)plane * HW + p0) * Cb;                    // np rows of Cb floats
    const int tid = threadIdx.x;

    if (!kUnpack) {
        for (int c = tid / kPix; c < Cb; c += kBlock / kPix) {
            const int p = tid % kPix;
            if (p < np) tile[c][p] = plain[(size_t)c * HW + p];
        }
        __syncthreads();
        for (int e = tid; e < np * Cb; e += kBlock) {
            const int p = e / Cb, c = e - p * Cb;
            blk[e] = tile[c][p];
        }
    } else {
        for (int e = tid; e < np * Cb; e += kBlock) {
            const int p = e / Cb, c = e - p * Cb;
            tile[c][p] = blk[e];
        }
        __syncthreads();
        for (int c = tid / kPix; c < Cb; c += kBlock / kPix) {
            const int p = tid % kPix;
            if (p < np) plain[(size_t)c * HW + p] = tile[c][p];
        }
    }
}

// Cb = 16 with a 16-byte aligned blocked tensor: 256 pixels x 16 channels per workgroup. A lane reads (writes) its
// pixel's 16 channel values with one coalesced 4-byte access per channel row, all in flight together, and the
// blocked side moves as whole float4s, 1 KB per wave instruction; LDS only transposes ([pixel][16 + 4 pad]).
constexpr int kPix16 = 256;

template <bool kUnpack>
__global__ void __launch_bounds__(kBlock) pack16(float *__restrict__ plain_base, float *__restrict__ blk_base, int C, int HW)
{
    __shared__ floatx4 tile[kPix16][5];
    const int nCb = C >> 4;
    const int plane = blockIdx.x;          // n * nCb + cb
    const int n = plane / nCb, cb = plane - n * nCb;
    const int p0 = blockIdx.y * kPix16;
    const int np = min(kPix16, HW - p0);
    float *plain = plain_base + ((size_t)n * C + (size_t)cb * 16) * HW + p0;
    floatx4 *blk = reinterpret_cast<floatx4 *>(blk_base + ((size_t)plane * HW + p0) * 16);
    const int t = threadIdx.x;
    if (!kUnpack) {
        if (t < np) {
            float v[16];
#pragma unroll
            for (int c = 0; c < 16; ++c) v[c] = __builtin_nontemporal_load(plain + (size_t)c * HW + t);
#pragma unroll
            for (int k = 0; k < 4; ++k) tile[t][k] = floatx4{v[4 * k], v[4 * k + 1], v[4 * k + 2], v[4 * k + 3]};
        }
        __syncthreads();
        for (int e = t; e < np * 4; e += kBlock) __builtin_nontemporal_store(tile[e >> 2][e & 3], blk + e);
    } else {
        for (int e = t; e < np * 4; e += kBlock) tile[e >> 2][e & 3] = __builtin_nontemporal_load(blk + e);
        __syncthreads();
        if (t < np) {
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const floatx4 v = tile[t][k];
#pragma unroll
                for (int c = 0; c < 4; ++c) __builtin_nontemporal_store(v[c], plain + (size_t)(4 * k + c) * HW + t);
            }
        }
    }
}

// Filters are packed once per network; one thread per blocked element.
__global__ void __launch_bounds__(kBlock) pack_filter_kernel(const float *__restrict__ oihw, float *__restrict__ blk,
                                                              int Co, int Ci, int kh, int kw, int Cob, int Cib)
{
    const size_t total = (size_t)Co * Ci * kh * kw;
    size_t e = (size_t)blockIdx.x * kBlock + threadIdx.x;
    if (e >= total) return;
    const size_t dst = e;
    const int co_in = (int)(e % Cob); e /= Cob;
    const int ci_in = (int)(e % Cib); e /= Cib;
    const int x = (int)(e % kw); e /= kw;
    const int y = (int)(e % kh); e /= kh;
    const int nCib = Ci / Cib;
    const int cib = (int)(e % nCib);
    const int cob = (int)(e / nCib);
    const int co = cob * Cob + co_in, ci = cib * Cib + ci_in;
    blk[dst] = oihw[(((size_t)co * Ci + ci) * kh + y) * kw + x];
}

}  // namespace

hipError_t launch_relu(const float *in, float *out, size_t n, hipStream_t s) { return launch_ew<false>(in, in, out, n, s); }
hipError_t launch_add(const float *a, const float *b, float *out, size_t n, hipStream_t s) { return launch_ew<true>(a, b, out, n, s); }

hipError_t launch_pack(const float *src, float *dst, int N, int C, int H, int W, int Cb, bool unpack, hipStream_t s)
{
    const int HW = H * W;
    if (Cb == 16 && HW >= 64 && ((uintptr_t)(unpack ? src : dst) & 15u) == 0) {
        const dim3 grid16((unsigned)(N * (C / 16)), (unsigned)((HW + kPix16 - 1) / kPix16));
        if (unpack) hipLaunchKernelGGL(pack16<true>, grid16, dim3(kBlock), 0, s, dst, const_cast<float *>(src), C, HW);
        else hipLaunchKernelGGL(pack16<false>, grid16, dim3(kBlock), 0, s, const_cast<float *>(src), dst, C, HW);
        return hipGetLastError();
    }
    const dim3 grid((unsigned)(N * (C / Cb)), (unsigned)((HW + kPix - 1) / kPix));
    // the source side is only read; the kernel takes both as plain pointers to share one body
    if (unpack)
        hipLaunchKernelGGL(pack_tile<true>, grid, dim3(kBlock), 0, s, dst, const_cast<float *>(src), C, HW, Cb);
    else
        hipLaunchKernelGGL(pack_tile<false>, grid, dim3(kBlock), 0, s, const_cast<float *>(src), dst, C, HW, Cb);
    return hipGetLastError();
}

hipError_t launch_pack_filter(const float *oihw, float *blk, int Co, int Ci, int kh, int kw, int Cob, int Cib,
                              hipStream_t s)
{
    const size_t total = (size_t)Co * Ci * kh * kw;
    hipLaunchKernelGGL(pack_filter_kernel, dim3((unsigned)((total + kBlock - 1) / kBlock)), dim3(kBlock), 0, s, oihw,
                       blk, Co, Ci, kh, kw, Cob, Cib);
    return hipGetLastError();
}

int device_cus()
{
    static const int n = [] {
        int dev = 0, cus = 0;
        if (hipGetDevice(&dev) != hipSuccess) return 256;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) return 256;
        return cus;
    }();
    return n;
}

}  // namespace small
