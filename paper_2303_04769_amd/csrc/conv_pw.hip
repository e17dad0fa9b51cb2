// Pointwise convolution (1x1 filter, stride 1, no padding; Table 1 row "Full Channel Reduction" with
// F_H = F_W = 1) on 16-channel blocks, for tensors with many pixels and a filter small enough to stay on the
// compute unit for the whole kernel (at most 128 x 128 channels: 64 KB).
//
// With few channels this layer moves 8..16 flop per byte: it is bound by HBM (64 channels) or close to it, and a
// tiled kernel that gives every workgroup one small tile spends its life in prologues (set-up, first-load latency).
// Here the grid is persistent (one workgroup of four waves per compute unit: one wave per SIMD) and every wavefront
// is autonomous:
//   - the filter is brought into LDS once per workgroup (global -> LDS loads with rows permuted, the layout of
//     conv_same.hip: matrix instruction r of a 16x16 slab reads LDS words 64 r + lane, conflict-free), then either
//     copied into registers (AREG) or read from LDS next to every matrix instruction (a quarter of the LDS bandwidth
//     at the full matrix rate);
//   - a task is 16 consecutive pixels (flattened over images) x COW output blocks; a wave walks tasks
//     w, w + W, w + 2W, ... (neighbouring waves work on neighbouring pixels at any time). The 16 pixels x NCIB input
//     blocks of a task (NCIB KB) go global -> LDS with one global_load_lds_dwordx4 per block into a ring of DEPTH + 1
//     stages that belongs to the wave alone, DEPTH tasks ahead of the matrix instructions; lane (pixel p, quad q)
//     then reads the 16 bytes of channels 4q..4q+3 of every block of pixel p -- the B operand of
//     v_mfma_f32_16x16x4_f32 (k slot q of instruction r = channel 4q + r) -- with ds_read_b128 (quads XOR-swizzled
//     by the per-lane source address of the load, conflict-free); the result (lane (p, q): output channels
//     4q..4q+3 of pixel p) is stored as it comes out of the accumulators, non-temporally.
//   No barrier after the filter has landed, no per-tile prologue. What is in flight is LDS memory, tracked with
//   hand-placed s_waitcnt vmcnt(n): every vector-memory instruction of the task loop is issued unconditionally, so the
//   number of instructions between a request and the wait for it is the same on every path, an operand wait never
//   also waits for the stores issued after the request, and a store has DEPTH tasks' time to complete. (Measured on
//   the 64-channel layer: with waits that also cover the stores, load, matrix and store time add up: 27 us.) The one pixel group that may be ragged (M % 16 pixels) is therefore not part of the loop: the last waves
//   of the grid take it afterwards with per-lane guards.
#include "small_internal.h"

#include <type_traits>

namespace small {

namespace {

constexpr int kPwMaxWaves = 8;              // wavefronts per workgroup, at most

struct PwArgs {
    const float *in;
    const float *filt;
    float *out;
    const float *res;
    const float *bn;          // EPI_BN: scale[0 .. Co) then shift[0 .. Co)
    int M, HW;                // pixels over all images, pixels per image
    int n_groups;             // ceil(M / 16)
    int epilogue;
    FastDiv dHW;
};

// NCIB / NCOB: input / output channel blocks of the layer; COW: output blocks per task (NCOB % COW == 0);
// AREG: the wave keeps its part of the filter (COW x NCIB slabs, 4 values per lane and slab) in registers;
// ADD: the result is accumulated onto the tensor `res` (residual connection folded into the STORE phase);
// DEPTH: tasks between the request of a task's operands and the matrix instructions that use them.
template <int NCIB, int NCOB, int COW, bool AREG, bool ADD, int DEPTH>
__global__ void __launch_bounds__(64 * kPwMaxWaves) pw16_stream(PwArgs a)
{
    constexpr int CSPLIT = NCOB / COW;
    constexpr int STAGE = NCIB * 1024;                      // bytes of one task's operands
    constexpr int RING = (DEPTH + 1) * STAGE;               // per wave
    static_assert(NCOB % COW == 0, "output blocks split evenly over tasks");     // (waves per workgroup % CSPLIT == 0: launcher)
    extern __shared__ floatx4 lds[];
    const unsigned lds_base = (unsigned)(uintptr_t)(__attribute__((address_space(3))) void *)lds;
    const float *lds_f = reinterpret_cast<const float *>(lds);
    const char *lds_c = reinterpret_cast<const char *>(lds);

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6);
    const int n_waves = (int)blockDim.x >> 6;
    const int lp = lane & 15, lq = lane >> 4;

    // ---- the filter: slab (cob, cib) -> LDS slab cob * NCIB + cib, rows permuted (LDS row 4r + q = channel 4q + r)
    {
        const int row = lane >> 2, ci = 4 * (row & 3) + (row >> 2);
        const unsigned voff = (unsigned)(ci * 16 + (lane & 3) * 4) * 4u;
        for (int slab = wave; slab < NCIB * NCOB; slab += n_waves)
            dma16(reinterpret_cast<const char *>(a.filt) + (size_t)slab * 1024, voff, lds_base + (unsigned)slab * 1024u);
    }

    // ---- work of this wave. Full rounds: in round k every wave has a task (pixel group g0 + k * gstride, output
    // blocks part * COW ..). The groups left over when the last round would keep only some of the waves busy are
    // cut finer instead: a unit is (pixel group, ONE output block), units go round-robin over all waves of the grid
    // (neighbouring waves share a pixel group), so the tail of the kernel is a quarter (64 channels) or an eighth of a
    // task long instead of a whole one. Units follow the tasks in the same operand pipeline.
    const int n_all = (int)gridDim.x * n_waves;             // waves of the grid
    const int gw = (int)blockIdx.x * n_waves + wave;
    const int part = gw % CSPLIT;
    const int gstride = n_all / CSPLIT;                     // pixel groups per round
    const int g0 = gw / CSPLIT;
    const int n_full = a.M >> 4;                            // pixel groups with all 16 pixels inside the tensor
    const int rounds = n_full / gstride;
    const int tail0 = rounds * gstride;                     // first pixel group of the tail
    const int n_units = (n_full - tail0) * NCOB;
    const int my_units = gw < n_units ? (n_units - gw + n_all - 1) / n_all : 0;
    const int n_items = rounds + my_units;                  // tasks, then units

    const char *in_c = reinterpret_cast<const char *>(a.in);
    char *out_c = reinterpret_cast<char *>(a.out);
    const char *res_c = reinterpret_cast<const char *>(a.res);
    const size_t plane = (size_t)a.HW * 64;                 // bytes of one channel block of one image
    const bool relu = (a.epilogue & EPI_RELU) != 0;

    // pixel group of this wave's item i (clamped to its last item; a wave without items: any valid group)
    auto group_of = [&](int i) -> int {
        const int ic = min(i, n_items - 1);
        if (ic < 0) return min(g0, a.n_groups - 1);
        return ic < rounds ? g0 + ic * gstride : tail0 + (gw + (ic - rounds) * n_all) / NCOB;
    };
    // byte offset of pixel px of group grp (block 0, first channel) in a tensor with nb channel blocks
    auto pixel_byte = [&](int grp, int px, int nb) -> unsigned {
        const int m = min(grp * 16 + px, a.M - 1);
        const int n = a.dHW.div(m), pix = m - n * a.HW;
        return (unsigned)(((n * nb) * a.HW + pix) * 64);
    };
    // ---- this wave's ring of operand stages, behind the filter. Stage layout per input block: [pixel e][quad], the
    // quad a load lane fetches chosen so that quad q of pixel e sits at position q ^ ((e >> 1) & 3).
    const unsigned ring = lds_base + (unsigned)(NCIB * NCOB * 1024 + wave * RING);
    const int le = lane >> 2;                                                   // load lane: pixel e, position lane & 3
    const unsigned l_quad = (unsigned)(((lane & 3) ^ ((le >> 1) & 3)) * 16);
    const char *r_ptr = lds_c + NCIB * NCOB * 1024 + wave * RING + (lp * 4 + (lq ^ ((lp >> 1) & 3))) * 16;
    auto request = [&](int grp, int stage) __attribute__((always_inline)) {
        const unsigned off = pixel_byte(grp, le, NCIB) + l_quad;
#pragma unroll
        for (int c = 0; c < NCIB; ++c)
            dma16(in_c + (size_t)c * plane, off, ring + (unsigned)(stage * STAGE + c * 1024));
    };

    // The first items' operands go out before the filter is awaited.
#pragma unroll
    for (int d = 0; d < DEPTH; ++d) request(group_of(d), d);

    wait_vmcnt<0>();
    __syncthreads();                                        // the filter is in LDS

    float areg[AREG ? COW : 1][AREG ? NCIB : 1][4];
    if constexpr (AREG) {
#pragma unroll
        for (int j = 0; j < COW; ++j)
#pragma unroll
            for (int c = 0; c < NCIB; ++c)
#pragma unroll
                for (int r = 0; r < 4; ++r) areg[j][c][r] = lds_f[((part * COW + j) * NCIB + c) * 256 + r * 64 + lane];
    }
    const float *a_lds = lds_f + (size_t)part * COW * NCIB * 256 + lane;

    using std::integral_constant;
    // acc[0 .. NJ) = filter blocks (NJ blocks from slab row fa_base, or the register copy) x the operands of `stage`
    auto reduce = [&](int stage, floatx4 *acc, auto nj, auto from_regs, const float *fa_base) __attribute__((always_inline)) {
        constexpr int NJ = decltype(nj)::value;
        floatx4 cur[NCIB];
#pragma unroll
        for (int c = 0; c < NCIB; ++c) cur[c] = *reinterpret_cast<const floatx4 *>(r_ptr + stage * STAGE + c * 1024);
#pragma unroll
        for (int j = 0; j < NJ; ++j) acc[j] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int c = 0; c < NCIB; ++c) {
            if constexpr (decltype(from_regs)::value) {
#pragma unroll
                for (int r = 0; r < 4; ++r)
#pragma unroll
                    for (int j = 0; j < NJ; ++j)
                        acc[j] = __builtin_amdgcn_mfma_f32_16x16x4f32(areg[j][c][r], cur[c][r], acc[j], 0, 0, 0);
            } else {
                float fa[NJ][4];
#pragma unroll
                for (int j = 0; j < NJ; ++j)
#pragma unroll
                    for (int r = 0; r < 4; ++r) fa[j][r] = fa_base[(j * NCIB + c) * 256 + r * 64];
#pragma unroll
                for (int r = 0; r < 4; ++r)
#pragma unroll
                    for (int j = 0; j < NJ; ++j)
                        acc[j] = __builtin_amdgcn_mfma_f32_16x16x4f32(fa[j][r], cur[c][r], acc[j], 0, 0, 0);
            }
        }
    };
    // a folded batch normalization: the parameters of this lane's four channels of output block cob
    const bool norm = (a.epilogue & EPI_BN) != 0;            // uniform
    auto bn_of = [&](int cob, floatx4 &sc, floatx4 &sh) __attribute__((always_inline)) {
        const float *bn_c = a.bn + cob * 16 + lq * 4;
        sc = *reinterpret_cast<const floatx4 *>(bn_c);
        sh = *reinterpret_cast<const floatx4 *>(bn_c + NCOB * 16);
    };
    floatx4 bn_sc[COW], bn_sh[COW];                          // of the tasks' output blocks, loaded once
#pragma unroll
    for (int j = 0; j < COW; ++j) {
        bn_sc[j] = bn_sh[j] = floatx4{0.f, 0.f, 0.f, 0.f};
        if (norm) bn_of(part * COW + j, bn_sc[j], bn_sh[j]);
    }
    auto finish = [&](floatx4 v, const char *res_p, floatx4 sc, floatx4 sh) __attribute__((always_inline)) -> floatx4 {
        if (norm) {
            v.x = fmaf(v.x, sc.x, sh.x); v.y = fmaf(v.y, sc.y, sh.y); v.z = fmaf(v.z, sc.z, sh.z); v.w = fmaf(v.w, sc.w, sh.w);
        }
        if constexpr (ADD) v += *reinterpret_cast<const floatx4 *>(res_p);
        v.x = (relu && !(v.x > 0.f)) ? 0.f : v.x; v.y = (relu && !(v.y > 0.f)) ? 0.f : v.y;
        v.z = (relu && !(v.z > 0.f)) ? 0.f : v.z; v.w = (relu && !(v.w > 0.f)) ? 0.f : v.w;
        return v;
    };
    // stores NJ consecutive output blocks from block `cob` on (sc, sh: their normalization parameters)
    auto store = [&](int grp, int cob, const floatx4 *acc, auto nj, const floatx4 *sc, const floatx4 *sh) __attribute__((always_inline)) {
        const unsigned o_off = pixel_byte(grp, lp, NCOB) + (unsigned)lq * 16u;
#pragma unroll
        for (int j = 0; j < decltype(nj)::value; ++j) {
            const size_t cb = (size_t)(cob + j) * plane + o_off;
            __builtin_nontemporal_store(finish(acc[j], res_c + cb, sc[j], sh[j]), reinterpret_cast<floatx4 *>(out_c + cb));
        }
    };
    // (a unit's output block changes from unit to unit: its parameters are loaded when it is stored)
    auto store_unit = [&](int grp, int cob, const floatx4 *acc) __attribute__((always_inline)) {
        floatx4 sc[1] = {floatx4{0.f, 0.f, 0.f, 0.f}}, sh[1] = {floatx4{0.f, 0.f, 0.f, 0.f}};
        if (norm) bn_of(cob, sc[0], sh[0]);
        store(grp, cob, acc, integral_constant<int, 1>{}, sc, sh);
    };

    // Item i works on stage i % (DEPTH + 1) and refills stage (i + DEPTH) % (DEPTH + 1), which item i - 1 has read
    // into registers. `newer`: vector-memory instructions issued between the requests of this item's operands and
    // the wait for them: the requests of the DEPTH items after it (always issued: beyond the wave's last item its
    // pixels again, unused) and the stores of the items before it that were issued since -- DEPTH * COW between tasks
    // in the steady state, fewer for the wave's first tasks (they stand outside the loop) and for units (one store
    // each: their waits count the requests only, which also waits for older stores; harmless in a tail).
    int i = 0, st = 0;                                      // item, its stage
    auto task = [&](int stage, auto newer) __attribute__((always_inline)) {
        const int sn = stage + DEPTH >= DEPTH + 1 ? stage - 1 : stage + DEPTH;
        request(group_of(i + DEPTH), sn);
        wait_vmcnt<decltype(newer)::value>();
        floatx4 acc[COW];
        reduce(stage, acc, integral_constant<int, COW>{}, integral_constant<bool, AREG>{}, a_lds);
        store(g0 + i * gstride, part * COW, acc, integral_constant<int, COW>{}, bn_sc, bn_sh);
        ++i;
    };
    static_assert(DEPTH >= 1 && DEPTH <= 3, "one to three items ahead");
    constexpr int steady = DEPTH * (NCIB + COW);
    static_assert(steady < 64, "vmcnt is a 6-bit counter");
    if (i < rounds) task(0, integral_constant<int, DEPTH * NCIB>{});
    if constexpr (DEPTH >= 2) { if (i == 1 && i < rounds) task(1, integral_constant<int, DEPTH * NCIB + COW>{}); }
    if constexpr (DEPTH >= 3) { if (i == 2 && i < rounds) task(2, integral_constant<int, DEPTH * NCIB + 2 * COW>{}); }
    st = i % (DEPTH + 1);
    while (i < rounds) {
        task(st, integral_constant<int, steady>{});
        st = st == DEPTH ? 0 : st + 1;
    }
    while (i < n_items) {
        const int sn = st + DEPTH >= DEPTH + 1 ? st - 1 : st + DEPTH;
        request(group_of(i + DEPTH), sn);
        wait_vmcnt<DEPTH * NCIB>();
        const int u = gw + (i - rounds) * n_all, cob = u % NCOB;
        floatx4 acc[1];
        reduce(st, acc, integral_constant<int, 1>{}, integral_constant<bool, false>{}, lds_f + (size_t)cob * NCIB * 256 + lane);
        store_unit(tail0 + u / NCOB, cob, acc);
        ++i;
        st = st == DEPTH ? 0 : st + 1;
    }
    wait_vmcnt<0>();                                        // the unused requests of the last items have landed

    // ---- the ragged group, if any: one output block per wave, the first waves of the grid
    if (n_full < a.n_groups)
    for (int cob = gw; cob < NCOB; cob += n_all) {
        request(n_full, 0);
        wait_vmcnt<0>();
        floatx4 acc[1];
        reduce(0, acc, integral_constant<int, 1>{}, integral_constant<bool, false>{}, lds_f + (size_t)cob * NCIB * 256 + lane);
        if (n_full * 16 + lp < a.M) store_unit(n_full, cob, acc);
    }
}

// PER_CU workgroups of four waves per compute unit: with 64 channels two (eight waves hide the load latency of a layer
// that is bound by HBM; measured 18.2 us against 19.6 with one), with 128 channels one (the 64 KB filter and the
// rings allow no more, and the layer is bound by the matrix pipe: one wave per SIMD keeps it busy).
template <int NCIB, int NCOB, int COW, bool AREG, bool ADD, int DEPTH, int PER_CU>
hipError_t launch_pw_cfg(const PwArgs &a, hipStream_t s)
{
    constexpr int waves = 4;
    constexpr size_t lds_bytes = (size_t)NCIB * NCOB * 1024 + (size_t)waves * (DEPTH + 1) * NCIB * 1024;
    static_assert(PER_CU * lds_bytes <= 160 * 1024, "LDS of a compute unit");
    static_assert(waves % (NCOB / COW) == 0, "the waves of a workgroup share the output blocks evenly");
    auto kern = pw16_stream<NCIB, NCOB, COW, AREG, ADD, DEPTH>;
    if (lds_bytes > 64 * 1024) {
        static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        if (attr != hipSuccess) return attr;
    }
    const long tasks = (long)a.n_groups * (NCOB / COW);
    long wgs = (long)PER_CU * device_cus();
    const long need = (tasks + waves - 1) / waves;
    if (wgs > need) wgs = need;
    hipLaunchKernelGGL(kern, dim3((unsigned)wgs), dim3(64 * waves), lds_bytes, s, a);
    return hipGetLastError();
}

}  // namespace

bool conv_pw_eligible(const LayerGeom &g)
{
    if (g.Cib != 16 || g.Cob != 16 || g.kh != 1 || g.kw != 1 || g.stride != 1 || g.pt || g.pl) return false;
    if (g.Ho != g.H || g.Wo != g.W) return false;
    const int nCib = g.Ci / 16, nCob = g.Co / 16;
    if (!((nCib == 4 && nCob == 4) || (nCib == 8 && nCob == 8))) return false;
    const size_t M = (size_t)g.N * g.H * g.W;
    // enough pixel groups for several tasks per wave, and 32-bit byte offsets
    return M >= (size_t)1 << 15 && M * (size_t)g.Ci < ((size_t)1 << 30) && M * (size_t)g.Co < ((size_t)1 << 30);
}

const char *conv_pw_kernel_name(const LayerGeom &g)
{
    return g.Ci == 64 ? "pw16_stream<4,4,4,1,1>" : "pw16_stream<8,8,4,0,1>";
}

hipError_t launch_conv_pw(const float *in, const float *filt, float *out, const float *res, const LayerGeom &g,
                          int epilogue, hipStream_t s, const float *bn)
{
    PwArgs a;
    a.in = in; a.filt = filt; a.out = out; a.res = (epilogue & EPI_ADD) ? res : out;
    a.bn = (epilogue & EPI_BN) ? bn : filt;
    a.HW = g.H * g.W;
    a.M = g.N * a.HW;
    a.n_groups = (a.M + 15) / 16;
    a.epilogue = epilogue;
    a.dHW = make_fastdiv(a.HW);
    const bool add = (epilogue & EPI_ADD) != 0;
    if (g.Ci == 64) return add ? launch_pw_cfg<4, 4, 4, true, true, 1, 2>(a, s) : launch_pw_cfg<4, 4, 4, true, false, 1, 2>(a, s);
    return add ? launch_pw_cfg<8, 8, 4, false, true, 1, 1>(a, s) : launch_pw_cfg<8, 8, 4, false, false, 1, 1>(a, s);
}

}  // namespace small
