// A run of pointwise layers in one kernel: fully connected layers on 1x1 images and 1x1 stride-1 convolutions,
// each optionally followed by ReLU (the dense-only autoencoder of Section "MLPerf:Tiny Inference Models" is one
// such run from its input to its output). A pointwise layer maps every pixel on its own, so a workgroup takes a
// tile of pixels through the whole run: the activations stay in LDS, only the filters stream in, and nothing
// but the run's input and its last output touches HBM. This is the abstract fused layer of the paper's
// "Conclusion & Future Directions" for the full-reduction class of Table 1 (F_H = F_W = 1).
//
// Per workgroup (8 waves): 16 * WM pixels. Wave w owns output channel block w of every layer. One reduction
// step covers one 16-channel input block: the wave's own 16 x 16 filter block (1 KB) is copied global -> LDS by
// the load unit into a ring private to the wave, STAGES - 1 steps ahead and across layer boundaries (filters do
// not depend on activations), so the waves only meet at the layer boundaries, where the activations change
// hands. The matrix-core operands:
//   A (filter):  lane (p = l % 16, q = l / 16) in MFMA r supplies filt[ci = 4q + r][co = p]; the copy stores
//                row ci = 4q + r of a block at LDS row 4r + q, so that one ds_read_b32 per r is conflict-free.
//   B (input):   lane (p, q) supplies channels 4q .. 4q + 3 of pixel p as one float4 (MFMA r takes element r).
//   D (output):  lane (p, q) receives channels 4q .. 4q + 3 of pixel p: exactly the B layout of the next layer.
// So a layer's results go to LDS as a plain dump of the accumulator registers ([channel block][pixel group][lane]
// float4, linear per wave) and come back as the next layer's B operand with no shuffle.
//
// Tensors with 8 channels (stored with an 8-channel block) may occur inside the run: their upper eight
// channels are carried as zeros in a 16-channel block, and the filter rows / columns that do not exist are
// read as duplicates of existing ones (finite values times zero).
#include "small_internal.h"

namespace small {
namespace {

constexpr int kSlabBytes = 8 * 1024;  // one ring stage: 8 waves x one 16 ci x 16 co filter block
constexpr int kWaves = 8;
constexpr int kThreads = kWaves * 64;

enum : int { KIND_16x16 = 0, KIND_COB8 = 1, KIND_CIB8 = 2 };

struct ChainLayerDev {
    const float *filt;
    int nCib, nCob, kind, relu;
};

struct ChainArgs {
    const float *in;
    float *out;
    int M, HW;            // pixels in all images, pixels per image
    int n_layers, n_slabs;
    int nCb_in, nCb_out;  // 16-channel blocks of the run's input and output tensors
    ChainLayerDev layer[kChainMaxLayers];
};

// A wave-uniform pointer the compiler may hold in vector registers, moved to scalar registers.
__device__ __forceinline__ const float *uniform(const float *p)
{
    const uintptr_t v = (uintptr_t)p;
    const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)v), hi = __builtin_amdgcn_readfirstlane((unsigned)(v >> 32));
    return (const float *)(((uintptr_t)hi << 32) | lo);
}

typedef const __attribute__((address_space(4))) ChainArgs *KernArgs;

// Prefetch cursor over the flat sequence of filter blocks this wave needs: (layer, input block) in order.
struct Cursor {
    const float *ptr;      // block to copy next
    int left;              // blocks left in the cursor's layer, this one included
    int layer;
    unsigned stride;       // floats between consecutive input blocks of one output block
    unsigned lane_off;     // per-lane byte offset inside a block for this layer's block shape
};

__device__ __forceinline__ void enter_layer(Cursor &c, KernArgs ka, int layer, int w, unsigned off16, unsigned off_cob8,
                                            unsigned off_cib8)
{
    const int nCib = ka->layer[layer].nCib, nCob = ka->layer[layer].nCob, kind = ka->layer[layer].kind;
    const int cob = w < nCob ? w : nCob - 1;      // waves without a block of their own copy the last one again
    c.stride = kind == KIND_16x16 ? 256u : 128u;
    c.ptr = ka->layer[layer].filt + (size_t)(cob * nCib) * c.stride;
    c.left = nCib;
    c.layer = layer;
    c.lane_off = kind == KIND_16x16 ? off16 : (kind == KIND_COB8 ? off_cob8 : off_cib8);
}

// One copy per wave and step, also past the last block (the cursor then stays on it), so the number of copies a
// wave has in flight is the same in every step.
__device__ __forceinline__ void issue_block(Cursor &c, KernArgs ka, int n_layers, int w, unsigned off16, unsigned off_cob8,
                                            unsigned off_cib8, unsigned lds_dst)
{
    dma16(uniform(c.ptr), c.lane_off, lds_dst);
    if (c.left > 1) {
        --c.left;
        c.ptr += c.stride;
    } else if (c.layer + 1 < n_layers) {
        enter_layer(c, ka, c.layer + 1, w, off16, off_cob8, off_cib8);
    }
}

// A fragments (one float per r) of the filter block at `slab`, B fragments (one float4 per 16-pixel group) at `actp`.
template <int WM>
__device__ __forceinline__ void load_operands(float (&af)[4], floatx4 (&b)[WM], const char *slab, unsigned a_step, const char *actp)
{
#pragma unroll
    for (int r = 0; r < 4; ++r) af[r] = *reinterpret_cast<const float *>(slab + r * a_step);
#pragma unroll
    for (int wm = 0; wm < WM; ++wm) b[wm] = *reinterpret_cast<const floatx4 *>(actp + wm * 1024);
}

template <int WM, int STAGES>
__global__ void __launch_bounds__(kThreads) dense_chain(ChainArgs args)
{
    // The layer table is indexed with run-time values: read it where it lies, in the kernel-argument segment
    // (constant address space, scalar loads), instead of through a private copy of the by-value argument.
    (void)args;
    const KernArgs ka = (KernArgs)__builtin_amdgcn_kernarg_segment_ptr();
    const float *const in = ka->in;
    float *const out = ka->out;
    const int M = ka->M, HW = ka->HW, n_layers = ka->n_layers, nCb_in = ka->nCb_in, nCb_out = ka->nCb_out;

    extern __shared__ floatx4 lds[];
    char *lds_c = reinterpret_cast<char *>(lds);
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int p = lane & 15, q = lane >> 4;
    // LDS byte addresses as the load unit takes them; lds_c + (x - ring) is the same byte for the compiler
    const unsigned ring = (unsigned)(uintptr_t)(__attribute__((address_space(3))) void *)lds;
    constexpr unsigned act_off = STAGES * kSlabBytes;
    const unsigned act = ring + act_off;

    // per-lane global byte offsets of the filter copy for the three block shapes
    const unsigned off16 = (unsigned)((4 * ((lane >> 2) & 3) + (lane >> 4)) * 64 + (lane & 3) * 16);
    const int l5 = lane & 31;
    const unsigned off_cob8 = (unsigned)((4 * ((l5 >> 1) & 3) + (l5 >> 3)) * 32 + (l5 & 1) * 16);
    const unsigned off_cib8 = (unsigned)((4 * ((lane >> 2) & 1) + (lane >> 4)) * 64 + (lane & 3) * 16);

    // input tile: channel block min(w, nCb_in - 1), WM groups of 16 pixels, straight into the activation buffer
    const int tile0 = (int)blockIdx.x * (16 * WM);
    {
        const int cb = w < nCb_in ? w : nCb_in - 1;
#pragma unroll
        for (int wm = 0; wm < WM; ++wm) {
            int m = tile0 + wm * 16 + p;
            m = m < M ? m : M - 1;
            const int n = m / HW, pix = m - n * HW;
            const unsigned off = (unsigned)((((size_t)n * nCb_in + cb) * HW + pix) * 64 + q * 16);
            dma16(uniform(in), off, act + (unsigned)((w * WM + wm) * 1024));
        }
    }
    Cursor c;
    enter_layer(c, ka, 0, w, off16, off_cob8, off_cib8);
#pragma unroll
    for (int s = 0; s < STAGES - 1; ++s)
        issue_block(c, ka, n_layers, w, off16, off_cob8, off_cib8, ring + (unsigned)s * kSlabBytes + (unsigned)w * 1024u);

    floatx4 acc[WM];
#pragma unroll
    for (int wm = 0; wm < WM; ++wm) acc[wm] = floatx4{0.f, 0.f, 0.f, 0.f};

    int s = 0;
    for (int l = 0; l < n_layers; ++l) {
        const int nCib = ka->layer[l].nCib, nCob = ka->layer[l].nCob, kind = ka->layer[l].kind, relu = ka->layer[l].relu;
        const bool mine = w < nCob;
        // LDS address of this lane's A element for r = 0 within a ring stage
        const unsigned a_lane = (unsigned)(w * 1024) + (kind == KIND_COB8 ? (unsigned)(q * 32 + (p & 7) * 4) : (unsigned)(lane * 4));
        const unsigned a_step = kind == KIND_COB8 ? 128u : 256u;
        if (l == 0) {
            wait_vmcnt<STAGES - 1>();   // the input tile copies of this wave have landed
            __syncthreads();            // ... and those of the other waves
        }
        for (int cib = 0; cib < nCib; ++cib, ++s) {
            wait_vmcnt<STAGES - 2>();   // this wave's filter block of step s has landed
            // the ring stage read in step s - 1 is free: this wave alone reads and refills its part
            issue_block(c, ka, n_layers, w, off16, off_cob8, off_cib8,
                        ring + (unsigned)((s + STAGES - 1) % STAGES) * kSlabBytes + (unsigned)w * 1024u);
            if (mine) {
                float af[4];
                floatx4 b[WM];
                load_operands<WM>(af, b, lds_c + (unsigned)(s % STAGES) * kSlabBytes + a_lane, a_step,
                                  lds_c + act_off + (cib * WM * 64 + lane) * 16);
#pragma unroll
                for (int r = 0; r < 4; ++r)
#pragma unroll
                    for (int wm = 0; wm < WM; ++wm)
                        acc[wm] = __builtin_amdgcn_mfma_f32_16x16x4f32(af[r], b[wm][r], acc[wm], 0, 0, 0);
            }
        }
        __syncthreads();   // every wave has read this layer's input: the activation buffer may be overwritten
        if (mine) {
            const bool last = l + 1 == n_layers;
#pragma unroll
            for (int wm = 0; wm < WM; ++wm) {
                floatx4 v = acc[wm];
                if (relu) {
#pragma unroll
                    for (int r = 0; r < 4; ++r) v[r] = v[r] > 0.f ? v[r] : 0.f;
                }
                if (kind == KIND_COB8 && q >= 2) v = floatx4{0.f, 0.f, 0.f, 0.f};
                if (last) {
                    const int m = tile0 + wm * 16 + p;
                    if (m < M) {
                        const int n = m / HW, pix = m - n * HW;
                        float *o = out + (((size_t)n * nCb_out + w) * HW + pix) * 16 + q * 4;
                        *reinterpret_cast<floatx4 *>(o) = v;
                    }
                } else {
                    *reinterpret_cast<floatx4 *>(lds_c + act_off + ((w * WM + wm) * 64 + lane) * 16) = v;
                }
                acc[wm] = floatx4{0.f, 0.f, 0.f, 0.f};
            }
        }
        __syncthreads();   // the next layer's input is complete
    }
    wait_vmcnt<0>();   // copies issued past the last block must land before the workgroup's LDS is released
}

template <int WM, int STAGES>
hipError_t launch_cfg(const ChainArgs &a, hipStream_t s)
{
    const size_t lds = (size_t)STAGES * kSlabBytes + (size_t)WM * 8 * 1024;
    const unsigned tiles = (unsigned)((a.M + 16 * WM - 1) / (16 * WM));
    if (lds >= 64 * 1024) {
        static hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void *>(dense_chain<WM, STAGES>),
                                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (attr != hipSuccess) return attr;
    }
    hipLaunchKernelGGL((dense_chain<WM, STAGES>), dim3(tiles), dim3(kThreads), lds, s, a);
    return hipGetLastError();
}

}  // namespace

bool chain_layer_eligible(int Ci, int Co, int Cib, int Cob)
{
    if (Ci <= 0 || Co <= 0 || Ci > 16 * kChainMaxBlocks || Co > 16 * kChainMaxBlocks) return false;
    const bool in16 = Cib == 16 && Ci % 16 == 0, in8 = Cib == 8 && Ci == 8;
    const bool out16 = Cob == 16 && Co % 16 == 0, out8 = Cob == 8 && Co == 8;
    return (in16 && out16) || (in16 && out8) || (in8 && out16);
}

hipError_t launch_dense_chain(const float *in, float *out, const ChainLayer *layers, int n_layers, long M, int HW,
                              hipStream_t s)
{
    ChainArgs a;
    a.in = in;
    a.out = out;
    a.M = (int)M;
    a.HW = HW;
    a.n_layers = n_layers;
    a.n_slabs = 0;
    a.nCb_in = layers[0].Ci / 16;
    a.nCb_out = layers[n_layers - 1].Co / 16;
    for (int i = 0; i < n_layers; ++i) {
        const ChainLayer &c = layers[i];
        ChainLayerDev &d = a.layer[i];
        d.filt = c.filt;
        d.nCib = c.Ci == 8 ? 1 : c.Ci / 16;
        d.nCob = c.Co == 8 ? 1 : c.Co / 16;
        d.kind = c.Co == 8 ? KIND_COB8 : (c.Ci == 8 ? KIND_CIB8 : KIND_16x16);
        d.relu = c.relu;
        a.n_slabs += d.nCib;
    }
    for (int i = n_layers; i < kChainMaxLayers; ++i) a.layer[i] = ChainLayerDev{nullptr, 0, 0, 0, 0};
    // pixels per workgroup: the largest tile that still gives every compute unit two workgroups
    // pixels per workgroup: the largest tile that still gives every compute unit two workgroups
    if (M >= 64L * 512) return launch_cfg<4, 4>(a, s);
    if (M >= 32L * 512) return launch_cfg<2, 4>(a, s);
    return launch_cfg<1, 4>(a, s);
}

}  // namespace small
