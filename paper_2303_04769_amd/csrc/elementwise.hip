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

// 16-channel blocks with a multiple of four pixels per plane: no LDS. A wave moves a tile of 64 pixels x 16 channels
// (4 KB): lane (r, g) holds channels 4r .. 4r + 3 of pixels 4g .. 4g + 3. On the plain side that is four 16-byte
// accesses (one per channel: four consecutive pixels of its row), on the blocked side four 16-byte accesses (one per
// pixel: its channel quad r); between the two lies a 4 x 4 transposition inside the lane's registers, i.e. nothing.
// Every access of a wave covers whole 64-byte (blocked) or 256-byte (plain) runs.
template <bool kUnpack>
__global__ void __launch_bounds__(kBlock) pack16_reg(float *__restrict__ plain_base, float *__restrict__ blk_base, int C, int HW,
                                                     int tiles_per_plane, int n_wave_tiles, FastDiv by_tiles, FastDiv by_nCb)
{
    const int wave_tile = (int)blockIdx.x * (kBlock / 64) + (int)(threadIdx.x >> 6);
    if (wave_tile >= n_wave_tiles) return;
    const int plane = by_tiles.div(wave_tile), tile = wave_tile - plane * tiles_per_plane;       // plane = n * nCb + cb
    const int nCb = C >> 4;
    const int n = by_nCb.div(plane), cb = plane - n * nCb;
    const int lane = threadIdx.x & 63, r = lane & 3, g = lane >> 2;
    const int p = tile * 64 + g * 4;                            // first of this lane's four pixels
    if (p >= HW) return;                                        // (HW is a multiple of 4: all four or none)
    float *plain = plain_base + ((size_t)n * C + (size_t)cb * 16 + 4 * r) * HW + p;
    float *blk = blk_base + ((size_t)plane * HW + p) * 16 + 4 * r;
    floatx4 v[4];
    if (!kUnpack) {
#pragma unroll
        for (int i = 0; i < 4; ++i) v[i] = __builtin_nontemporal_load(reinterpret_cast<const floatx4 *>(plain + (size_t)i * HW));
#pragma unroll
        for (int j = 0; j < 4; ++j)
            __builtin_nontemporal_store(floatx4{v[0][j], v[1][j], v[2][j], v[3][j]}, reinterpret_cast<floatx4 *>(blk + j * 16));
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) v[j] = __builtin_nontemporal_load(reinterpret_cast<const floatx4 *>(blk + j * 16));
#pragma unroll
        for (int i = 0; i < 4; ++i)
            __builtin_nontemporal_store(floatx4{v[0][i], v[1][i], v[2][i], v[3][i]}, reinterpret_cast<floatx4 *>(plain + (size_t)i * HW));
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
    if (Cb == 16 && HW % 4 == 0 && ((((uintptr_t)src | (uintptr_t)dst) & 15u) == 0)) {
        const int tiles = (HW + 63) / 64;
        const long waves = (long)N * (C / 16) * tiles;
        const unsigned grid = (unsigned)((waves + kBlock / 64 - 1) / (kBlock / 64));
        if (unpack)
            hipLaunchKernelGGL(pack16_reg<true>, dim3(grid), dim3(kBlock), 0, s, dst, const_cast<float *>(src), C, HW, tiles,
                               (int)waves, make_fastdiv(tiles), make_fastdiv(C / 16));
        else
            hipLaunchKernelGGL(pack16_reg<false>, dim3(grid), dim3(kBlock), 0, s, const_cast<float *>(src), dst, C, HW, tiles,
                               (int)waves, make_fastdiv(tiles), make_fastdiv(C / 16));
        return hipGetLastError();
    }
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
