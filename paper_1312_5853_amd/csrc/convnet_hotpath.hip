// HIP kernels (gfx950 / CDNA4) and C-ABI entry points of the convolution hot
// path: forward, backward-data and backward-filter of a convolutional layer as
// implicit GEMMs on the fp32 matrix cores, plus the ReLU / max-pool glue of
// the five-layer stack.  Signatures and conventions are documented in
// include/convnet_hotpath.h.
//
// GEMM views (NCHW activations, KCRS filters, P x Q output extent):
//   forward         y  [K      x N*P*Q] = w  [K x C*R*S]  *  im2col(x)  [C*R*S x N*P*Q]
//   backward-data   dx [C      x N*H*W] = w' [C x K*R*S]  *  col2im-gather(dy)
//   backward-filter dw [K      x C*R*S] = dy [K x N*P*Q]  *  im2col(x)^T, split over N*P*Q
// The im2col matrices are never materialised in HBM: each work-group gathers
// the 16-deep slice it needs straight from the NCHW tensor into LDS.
#include <hip/hip_runtime.h>

#include <stdio.h>
#include <algorithm>
#include <mutex>
#include <type_traits>
#include <stdlib.h>
#include <string.h>

#include "../../include/convnet_hotpath.h"
#include "plan.h"

using namespace convnet;

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// Scratch of conv_bwd_filter_noalloc: one copy per GPU, held until the process ends.  In host code this name is only
// a handle for hipGetSymbolAddress; kernels and memory calls take the address that call returns.
static __device__ __align__(256) unsigned char scratch[CONV_NOALLOC_SCRATCH_BYTES];

namespace {

constexpr int kThreads = 256;        // 4 wavefronts of 64
constexpr int kPitch = kChunk + 4;   // LDS row pitch (floats): 16 lanes x b128 cover all 64 banks once
constexpr int kInvalidTap = -(1 << 29);

__device__ __forceinline__ int uniform(int v) { return __builtin_amdgcn_readfirstlane(v); }

#include "device_common.h"
#include "conv_colgemm_kernels.h"
#include "conv_bf16_dma_kernels.h"
#include "conv_wgrad_rows_kernels.h"
#include "conv_wgrad_kernels.h"
#include "fc_kernels.h"
#include "glue_kernels.h"

// ---------------------------------------------------------------------------
// Host side
// ---------------------------------------------------------------------------
thread_local char g_hip_error[256] = "";

int hip_fail(hipError_t e)
{
    snprintf(g_hip_error, sizeof(g_hip_error), "%s", hipGetErrorString(e));
    return kErrHip;
}

int check_launch()
{
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? kStatusOk : hip_fail(e);
}

bool aligned(const void *p, size_t a) { return ((uintptr_t)p % a) == 0; }


// Tiles are spread evenly over the 8 XCDs (32 CUs each).  When that gives at
// most `cap` <= 3 work-groups per CU, extra dynamic LDS is requested so that no
// CU can hold more than `cap`: the dispatcher is then forced to balance, and
// the launch ends when the evenly loaded CUs end instead of waiting for a CU
// that was handed one work-group more.
struct GridPlan { int tiles_per_xcd, grid, dyn_lds; };

GridPlan plan_grid(int tiles, int static_lds)
{
    GridPlan g;
    g.tiles_per_xcd = ceil_div(tiles, 8);
    g.grid = 8 * g.tiles_per_xcd;
    int cap = ceil_div(g.tiles_per_xcd, 32);
    int total = static_lds;
    if (cap == 3) total = 52 * 1024;
    else if (cap <= 2) total = 64 * 1024;
    g.dyn_lds = total > static_lds ? total - static_lds : 0;
    return g;
}

template <int GATHER>
void launch_colgemm(const TileShape &t, const ColGemmArgs &a, const GridPlan &g, hipStream_t st)
{
    const dim3 grid(g.grid), block(kThreads);
    if (t.TM == 2 && t.TN == 2) hipLaunchKernelGGL((colgemm_kernel<2, 2, 2, 2, GATHER>), grid, block, g.dyn_lds, st, a);
    else if (t.TM == 3) hipLaunchKernelGGL((colgemm_kernel<3, 1, 1, 4, GATHER>), grid, block, g.dyn_lds, st, a);
    else if (t.TM == 2) hipLaunchKernelGGL((colgemm_kernel<2, 1, 1, 4, GATHER>), grid, block, g.dyn_lds, st, a);
    else hipLaunchKernelGGL((colgemm_kernel<1, 2, 1, 4, GATHER>), grid, block, g.dyn_lds, st, a);
}

template <typename Kern>
void launch_dyn(Kern kern, const ColGemmFastArgs &a, int grid, int lds, hipStream_t st)
{
    // more than 64 KB of dynamic LDS has to be allowed per kernel
    if (lds > 64 * 1024)
        (void)hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                  160 * 1024);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(kThreads), lds, st, a);
}

void launch_colgemm_fast(const TileShape &t, int kc, const ColGemmFastArgs &a, const GridPlan &g, hipStream_t st)
{
    const int need = 2 * (t.bm() + t.bn()) * (kc + 4) * 4;
    const int lds = need + g.dyn_lds;
    if (t.mfma == 16) launch_dyn(colgemm_rows48_kernel, a, g.grid, lds, st);
    else if (t.TM == 2 && t.TN == 2) launch_dyn(colgemm_fast_kernel<2, 2, 2, 2, 16>, a, g.grid, lds, st);
    else if (t.TM == 3) launch_dyn(colgemm_fast_kernel<3, 1, 1, 4, 16>, a, g.grid, lds, st);
    else if (t.TM == 2) launch_dyn(colgemm_fast_kernel<2, 1, 1, 4, 16>, a, g.grid, lds, st);
    else launch_dyn(colgemm_fast_kernel<1, 2, 1, 4, 16>, a, g.grid, lds, st);
}

template <typename TI, typename TO>
void launch_patch_typed(int tm, const PatchArgs &a, int grid, int lds, hipStream_t st)
{
    const void *k = tm == 1 ? (const void *)colgemm_patch_kernel<1, TI, TO>
                  : tm == 2 ? (const void *)colgemm_patch_kernel<2, TI, TO>
                  : tm == 3 ? (const void *)colgemm_patch_kernel<3, TI, TO>
                            : (const void *)colgemm_patch_kernel<4, TI, TO>;
    if (lds > 64 * 1024) (void)hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (tm == 1) hipLaunchKernelGGL((colgemm_patch_kernel<1, TI, TO>), dim3(grid), dim3(kThreads), lds, st, a);
    else if (tm == 2) hipLaunchKernelGGL((colgemm_patch_kernel<2, TI, TO>), dim3(grid), dim3(kThreads), lds, st, a);
    else if (tm == 3) hipLaunchKernelGGL((colgemm_patch_kernel<3, TI, TO>), dim3(grid), dim3(kThreads), lds, st, a);
    else hipLaunchKernelGGL((colgemm_patch_kernel<4, TI, TO>), dim3(grid), dim3(kThreads), lds, st, a);
}

// in_bf16 / out_bf16: element types of x and y
void launch_patch(int tm, const PatchArgs &a, int grid, int lds, bool in_bf16, bool out_bf16, hipStream_t st)
{
    if (!in_bf16) launch_patch_typed<float, float>(tm, a, grid, lds, st);
    else if (!out_bf16) launch_patch_typed<unsigned short, float>(tm, a, grid, lds, st);
    else launch_patch_typed<unsigned short, unsigned short>(tm, a, grid, lds, st);
}

template <int KC>
void launch_colgemm_bf16_kc(const TileShape &t, const ColGemmFastArgs &a, const GridPlan &g, hipStream_t st)
{
    const int lds = 2 * (t.bm() + t.bn()) * (KC * 2 + 16) + g.dyn_lds;
    if (t.TM == 2 && t.TN == 2) launch_dyn(colgemm_bf16_kernel<2, 2, 2, 2, KC>, a, g.grid, lds, st);
    else if (t.TM == 3) launch_dyn(colgemm_bf16_kernel<3, 1, 1, 4, KC>, a, g.grid, lds, st);
    else if (t.TM == 2) launch_dyn(colgemm_bf16_kernel<2, 1, 1, 4, KC>, a, g.grid, lds, st);
    else launch_dyn(colgemm_bf16_kernel<1, 2, 1, 4, KC>, a, g.grid, lds, st);
}

// channels per step of the bf16 kernel: the largest of 64, 48, 32, 16 that divides the channel count
int bf16_step_channels(int channels)
{
    return channels % 64 == 0 ? 64 : channels % 48 == 0 ? 48 : channels % 32 == 0 ? 32 : 16;
}

void launch_colgemm_bf16(const TileShape &t, int kc, const ColGemmFastArgs &a, const GridPlan &g, hipStream_t st)
{
    if (kc == 64) launch_colgemm_bf16_kc<64>(t, a, g, st);
    else if (kc == 48) launch_colgemm_bf16_kc<48>(t, a, g, st);
    else if (kc == 32) launch_colgemm_bf16_kc<32>(t, a, g, st);
    else launch_colgemm_bf16_kc<16>(t, a, g, st);
}

int grid1d(int64_t n, int block) { return (int)((n + block - 1) / block); }

template <typename Kern>
void launch_dma(Kern kern, const ColGemmDmaArgs &a, int grid, int lds, hipStream_t st, int threads = kThreads)
{
    if (lds > 64 * 1024)
        (void)hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                  160 * 1024);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(threads), lds, st, a);
}

// bf16 forward / stride-1 backward-data on the direct-to-LDS kernel: one preparation launch (padded channel-blocked
// activations + swizzled filters), then the contraction
int run_colgemm_dma(int op, const void *act, const void *w, void *out, const Problem &pb, const Plan &pl, void *ws,
                    hipStream_t st, const Epilogue *ep, bool *ep_applied)
{
    char *wsb = static_cast<char *>(ws);
    const bool fwd = op == kOpFwd;
    const int Cr = fwd ? pb.C : pb.K, RS = pb.R * pb.S, kc = pl.dma_kc;
    const int LH = fwd ? pb.H : pb.P, LW = fwd ? pb.W : pb.Q;
    DmaPrepArgs q;
    q.src = static_cast<const unsigned short *>(act);
    q.xb = reinterpret_cast<u32x4 *>(wsb + pl.xb_off);
    q.N = pb.N; q.CB = Cr / 16; q.LH = LH; q.LW = LW; q.Hp = pl.dma_hp; q.Wp = pl.dma_wp;
    q.pad_h = pl.dma_ph; q.pad_w = pl.dma_pw;
    q.src_bs = fwd ? pb.x_bs : pb.y_bs;
    const int64_t positions = (int64_t)pb.N * q.CB * q.Hp * q.Wp;
    // plane groups through LDS where they are 16-byte aligned and fit 64 KB; else one thread per position
    const int plane_lds = 32 * LH * LW;
    q.xb_planes = (q.src_bs % 8 == 0 && plane_lds <= 64 * 1024) ? 1 : 0;
    q.xb_blocks = q.xb_planes ? pb.N * q.CB : grid1d(positions, 256);
    q.w = static_cast<const unsigned short *>(w);
    q.wt = reinterpret_cast<unsigned short *>(wsb + pl.wt_off);
    q.M = pl.M; q.Mpad = pl.Mpad; q.cblocks = Cr / kc; q.RS = RS; q.C = pb.C; q.transposed = fwd ? 0 : 1; q.kc = kc;
    q.div_wp = make_fastdiv((uint32_t)q.Wp);
    q.div_hp = make_fastdiv((uint32_t)q.Hp);
    q.div_cb = make_fastdiv((uint32_t)q.CB);
    const int64_t wt_elems = (int64_t)pl.Mpad * Cr * RS;
    hipLaunchKernelGGL(bf16_dma_prepare, dim3(q.xb_blocks + grid1d(wt_elems / 8, 256)), dim3(256),
                       q.xb_planes ? plane_lds : 0, st, q);
    int rc = check_launch();
    if (rc != kStatusOk) return rc;

    ColGemmDmaArgs a;
    a.At = q.wt; a.xb = q.xb; a.dst = out; a.part = nullptr;
    a.M = pl.M; a.Mpad = pl.Mpad;
    a.OH = fwd ? pb.P : pb.H; a.OW = fwd ? pb.Q : pb.W; a.mul = fwd ? pb.stride : 1;
    a.ncols = pb.N * a.OH * a.OW;
    a.Wp = q.Wp; a.cb_bytes = q.Hp * q.Wp * 32; a.n_bytes = q.CB * a.cb_bytes;
    a.R = pb.R; a.S = pb.S; a.sign = fwd ? 1 : -1;
    a.cblocks = Cr / kc;
    a.dst_bs = (int)(fwd ? pb.y_bs : pb.x_bs); a.out_bf16 = pb.out_bf16;
    a.dst_small = (int64_t)pb.N * a.dst_bs * 2 < ((int64_t)1 << 31) ? 1 : 0;
    a.mtiles = pl.Mpad / pl.tile.bm();
    a.ntiles = ceil_div(a.ncols, pl.tile.bn());
    a.ksplit = 1; a.steps_per_split = a.cblocks * RS;
    a.epi_on = ep != nullptr;
    a.epi = ep ? *ep : Epilogue{};
    *ep_applied = a.epi_on;
    a.div_plane = make_fastdiv((uint32_t)(a.OH * a.OW));
    a.div_ow = make_fastdiv((uint32_t)a.OW);
    a.div_rs = make_fastdiv((uint32_t)RS);
    a.div_s = make_fastdiv((uint32_t)pb.S);
    a.tiles_per_xcd = ceil_div(a.mtiles * a.ntiles, 8);
    const int grid = 8 * a.tiles_per_xcd;
    const int lds = 3 * (pl.tile.bm() + pl.tile.bn()) * kc * 2;
    const int tn = pl.tile.TN;
    // one work-group per CU (64-channel steps): eight waves, two per SIMD, so that a wave's waits (fragment reads,
    // the barrier) leave the matrix pipe to the other; two work-groups per CU: four waves each
    if (tn == 4 && kc == 64) launch_dma(colgemm_bf16_dma_kernel<2, 2, 2, 4, 64, 1>, a, grid, lds, st, 512);
    else if (tn == 4) launch_dma(colgemm_bf16_dma_kernel<2, 4, 2, 2, 32, 2>, a, grid, lds, st);
    else if (tn == 3 && kc == 64) launch_dma(colgemm_bf16_dma_kernel<1, 3, 4, 2, 64, 1>, a, grid, lds, st, 512);
    else if (tn == 3) launch_dma(colgemm_bf16_dma_kernel<2, 3, 2, 2, 32, 2>, a, grid, lds, st);
    else if (kc == 64) launch_dma(colgemm_bf16_dma_kernel<2, 2, 2, 2, 64, 1>, a, grid, lds, st);
    else launch_dma(colgemm_bf16_dma_kernel<2, 2, 2, 2, 32, 2>, a, grid, lds, st);
    return check_launch();
}

constexpr int kNotTaken = 1;          // a specialised path declined the shape: the caller goes on to the general one

// Few-channel forward with bf16 inputs on the bf16 matrix instruction (conv_patch_bf16_kernel); kNotTaken where its
// alignment or size conditions do not hold.
template <int TN, typename TO>
const void *patch_bf16_kernel(int tm)
{
    return tm == 1 ? (const void *)conv_patch_bf16_kernel<1, TN, TO> : tm == 2 ? (const void *)conv_patch_bf16_kernel<2, TN, TO>
         : tm == 3 ? (const void *)conv_patch_bf16_kernel<3, TN, TO> : (const void *)conv_patch_bf16_kernel<4, TN, TO>;
}

int run_patch_bf16(const void *x, const void *w, void *out, const Problem &pb, const Plan &pl, void *ws,
                   hipStream_t st, const Epilogue *ep, bool *ep_applied)
{
    const int tm = pl.patch_tm, mpad = tm * 32;
    if (pb.S > 16 || pb.stride % 4 != 0 || pb.pad % 2 != 0 || pb.W % 8 != 0 || pb.x_bs % 8 != 0 || pl.M > mpad)
        return kNotTaken;
    if ((int64_t)pb.N * pb.y_bs * 2 >= ((int64_t)1 << 31)) return kNotTaken;     // 32-bit byte offsets into a bf16 output
    const int need_w = std::max(pb.pad + pb.W, (pb.Q - 1) * pb.stride + 16);
    const int wp = round_up(need_w, 4);
    const int nslices = pb.C * pb.R;
    const int64_t fbytes = (int64_t)nslices * mpad * 32;
    if (fbytes > (int64_t)pl.wt_bytes) return kNotTaken;
    // 256 positions per tile (each filter fragment read from LDS feeds two matrix instructions) where the tile's
    // input rows fit beside the filters, else 128
    int tn = 0, nr = 0;
    int64_t lds = 0;
    for (int t = tm <= 3 ? 2 : 1; t >= 1 && !tn; --t) {
        const int span = std::min((pb.Q + 128 * t - 2) / pb.Q, pb.P - 1);     // output rows a tile can straddle, minus one
        const int rows = span * pb.stride + pb.R;
        const int64_t bytes = fbytes + (int64_t)pb.C * rows * wp * 2;
        const int64_t pieces = (int64_t)pb.C * rows * (pb.W / 8);
        if (bytes <= 159 * 1024 && pieces <= kPatchBf16Pieces(t) * kThreads) { tn = t; nr = rows; lds = bytes; }
    }
    if (!tn) return kNotTaken;
    char *wsb = static_cast<char *>(ws);
    unsigned short *ft = reinterpret_cast<unsigned short *>(wsb + pl.wt_off);
    hipLaunchKernelGGL(relayout_filters_rows_bf16, dim3(grid1d(fbytes / 2, 256)), dim3(256), 0, st,
                       static_cast<const unsigned short *>(w), ft, pl.M, mpad, pb.C, pb.R, pb.S);
    PatchBf16Args a;
    a.Ft = ft; a.x = static_cast<const unsigned short *>(x); a.y = out;
    a.M = pl.M; a.Mpad = mpad; a.nslices = nslices;
    a.C = pb.C; a.H = pb.H; a.W = pb.W; a.R = pb.R; a.stride = pb.stride; a.pad = pb.pad;
    a.P = pb.P; a.Q = pb.Q; a.PQ = pb.P * pb.Q; a.NR = nr; a.WP = wp;
    a.x_bs = (int)pb.x_bs; a.y_bs = (int)pb.y_bs;
    a.jtiles = ceil_div(a.PQ, 128 * tn); a.ntiles = pb.N * a.jtiles;
    a.epi_on = ep != nullptr;
    a.epi = ep ? *ep : Epilogue{};
    *ep_applied = a.epi_on;
    a.div_q = make_fastdiv((uint32_t)pb.Q);
    a.div_j = make_fastdiv((uint32_t)a.jtiles);
    a.div_nr = make_fastdiv((uint32_t)nr);
    a.div_wv = make_fastdiv((uint32_t)(pb.W / 8));
    const int grid = std::min(a.ntiles, 256);
    const void *k = pb.out_bf16 ? (tn == 2 ? patch_bf16_kernel<2, unsigned short>(tm) : patch_bf16_kernel<1, unsigned short>(tm))
                                : (tn == 2 ? patch_bf16_kernel<2, float>(tm) : patch_bf16_kernel<1, float>(tm));
    (void)hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    void *args[] = {&a};
    hipError_t e = hipLaunchKernel(k, dim3(grid), dim3(kThreads), args, (size_t)lds, st);
    if (e != hipSuccess) return hip_fail(e);
    return check_launch();
}

// dw[k][c][rs] from the split partials part[split][k][rs*C + c] of `groups` columns (K, C per column)
int launch_finish_wgrad(const float *part, float *dw, int K, int C, int RS, int nsplit, int groups, hipStream_t st)
{
    const int ncols = RS * C;
    if (C % 4 == 0 && reinterpret_cast<uintptr_t>(part) % 16 == 0) {
        const int count = groups * K * (ncols / 4);
        hipLaunchKernelGGL(finish_wgrad_x4, dim3(grid1d(count, 256)), dim3(256), 0, st, part, dw, K, C, RS, nsplit, groups,
                           make_fastdiv((uint32_t)(K * (ncols / 4))), make_fastdiv((uint32_t)(ncols / 4)),
                           make_fastdiv((uint32_t)C));
    } else {
        const int count = groups * K * ncols;
        hipLaunchKernelGGL(finish_wgrad, dim3(grid1d(count, 256)), dim3(256), 0, st, part, dw, K, C, RS, nsplit, groups,
                           make_fastdiv((uint32_t)(K * ncols)), make_fastdiv((uint32_t)ncols), make_fastdiv((uint32_t)C));
    }
    return check_launch();
}

template <typename TI>
void launch_wgrad_typed(const TileShape &t, const WgradArgs &a, int grid, hipStream_t st)
{
    const dim3 g(grid), b(kThreads);
    if (t.TM == 2 && t.TN == 2) hipLaunchKernelGGL((wgrad_kernel<2, 2, 2, 2, TI>), g, b, 0, st, a);
    else if (t.TM == 3) hipLaunchKernelGGL((wgrad_kernel<3, 1, 1, 4, TI>), g, b, 0, st, a);
    else if (t.TM == 2) hipLaunchKernelGGL((wgrad_kernel<2, 1, 1, 4, TI>), g, b, 0, st, a);
    else hipLaunchKernelGGL((wgrad_kernel<1, 2, 1, 4, TI>), g, b, 0, st, a);
}

void launch_wgrad(const TileShape &t, const WgradArgs &a, int grid, bool in_bf16, hipStream_t st)
{
    if (in_bf16) launch_wgrad_typed<unsigned short>(t, a, grid, st);
    else launch_wgrad_typed<float>(t, a, grid, st);
}

constexpr int kWgradBf16Depth = 32;     // reduction positions per step of the bf16 backward-filter kernel

void launch_wgrad_bf16(const TileShape &t, const WgradFastArgs &a, int grid, int lds, hipStream_t st)
{
    constexpr int KJ = kWgradBf16Depth;
    const void *k = (t.TM == 2 && t.TN == 2) ? (const void *)wgrad_bf16_kernel<2, 2, 2, 2, KJ>
                  : t.TM == 3 ? (const void *)wgrad_bf16_kernel<3, 1, 1, 4, KJ>
                              : (const void *)wgrad_bf16_kernel<2, 1, 1, 4, KJ>;
    if (lds > 64 * 1024) (void)hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    const dim3 g(grid), b(kThreads);
    if (t.TM == 2 && t.TN == 2) hipLaunchKernelGGL((wgrad_bf16_kernel<2, 2, 2, 2, KJ>), g, b, lds, st, a);
    else if (t.TM == 3) hipLaunchKernelGGL((wgrad_bf16_kernel<3, 1, 1, 4, KJ>), g, b, lds, st, a);
    else hipLaunchKernelGGL((wgrad_bf16_kernel<2, 1, 1, 4, KJ>), g, b, lds, st, a);
}

void launch_wgrad_fast(const TileShape &t, const WgradFastArgs &a, const GridPlan &g, hipStream_t st)
{
    const dim3 grid(g.grid), block(kThreads);
    if (t.TM == 2 && t.TN == 2) hipLaunchKernelGGL((wgrad_fast_kernel<2, 2, 2, 2>), grid, block, g.dyn_lds, st, a);
    else if (t.TM == 3) hipLaunchKernelGGL((wgrad_fast_kernel<3, 1, 1, 4>), grid, block, g.dyn_lds, st, a);
    else if (t.TM == 2) hipLaunchKernelGGL((wgrad_fast_kernel<2, 1, 1, 4>), grid, block, g.dyn_lds, st, a);
    else hipLaunchKernelGGL((wgrad_fast_kernel<1, 2, 1, 4>), grid, block, g.dyn_lds, st, a);
}

// Common front end of the three passes: checks, plan, workspace carving.
int prepare(int op, const void *a, const void *b, void *out, int N, int C, int H, int W, int K, int R, int S,
            int stride, int pad, int64_t x_bs, int64_t y_bs, int dtype, void *ws, size_t ws_bytes,
            Problem &pb, Plan &pl)
{
    if (!a || !b || !out) return kErrInvalidArg;
    int rc = make_problem(pb, N, C, H, W, K, R, S, stride, pad, x_bs, y_bs, dtype);
    if (rc != kStatusOk) return rc;
    if (!aligned(a, 16) || !aligned(b, 16) || !aligned(out, 16)) return kErrMisaligned;
    pl = make_plan(op, pb);
    if (pl.total > 0) {
        if (!ws || ws_bytes < pl.total) return kErrWorkspace;
        if (!aligned(ws, 256)) return kErrMisaligned;
    }
    return kStatusOk;
}

// fp32 view of an input: the caller's tensor, or (widen, as the plan decided) a dense fp32 copy of `batch` samples of
// `sample` elements that lie `*bs` elements apart; *bs becomes the copy's stride.
const float *as_f32(bool widen, const void *src, int batch, int64_t sample, int64_t *bs, char *ws, const Plan &pl,
                    int slot, hipStream_t st)
{
    if (!widen) return static_cast<const float *>(src);
    float *dst = reinterpret_cast<float *>(ws + pl.cvt_off[slot]);
    const int64_t count = batch * sample;
    hipLaunchKernelGGL(widen_bf16, dim3(grid1d(count, 256)), dim3(256), 0, st,
                       static_cast<const unsigned short *>(src), dst, count, sample, *bs);
    *bs = sample;
    return dst;
}

int run_colgemm_f32out(int op, const void *act, const void *w, void *out, const Problem &caller_pb, const Plan &pl,
                       void *ws, hipStream_t st, const Epilogue *ep, bool *ep_applied);

// The epilogue as a pass of its own over out[N][rows][plane] (element type fp32 or bf16)
int run_epilogue_pass(void *out, bool out_bf16, int64_t out_bs, const Epilogue &e, int N, int rows, int plane,
                      hipStream_t st)
{
    const int per_sample = rows * plane;
    const int64_t total = (int64_t)N * per_sample;
    const FastDiv ds = make_fastdiv((uint32_t)per_sample), dp = make_fastdiv((uint32_t)plane);
    if (out_bf16)
        hipLaunchKernelGGL(epilogue_inplace<unsigned short>, dim3(grid1d(total, 256)), dim3(256), 0, st,
                           static_cast<unsigned short *>(out), out_bs, e, total, per_sample, ds, dp);
    else
        hipLaunchKernelGGL(epilogue_inplace<float>, dim3(grid1d(total, 256)), dim3(256), 0, st,
                           static_cast<float *>(out), out_bs, e, total, per_sample, ds, dp);
    return check_launch();
}

// Forward / backward-data.  The bf16 kernels write a bf16 destination themselves; for the other paths it is
// produced from a dense fp32 result in the workspace.  An epilogue (ep != null) is applied by the kernel that stores
// the final sums where that kernel can, else by a pass over the fp32 result.
int run_colgemm(int op, const void *act, const void *w, void *out, const Problem &pb, const Plan &pl, void *ws,
                hipStream_t st, const Epilogue *ep = nullptr)
{
    const int rows = op == kOpFwd ? pb.K : pb.C;
    const int plane = op == kOpFwd ? pb.P * pb.Q : pb.H * pb.W;
    bool applied = false;
    if (!pb.out_bf16 || pl.stage_bytes == 0) {
        int rc = run_colgemm_f32out(op, act, w, out, pb, pl, ws, st, ep, &applied);
        if (rc != kStatusOk || !ep || applied) return rc;
        return run_epilogue_pass(out, pb.out_bf16, op == kOpFwd ? pb.y_bs : pb.x_bs, *ep, pb.N, rows, plane, st);
    }
    Problem q = pb;
    q.out_bf16 = false;
    const int64_t sample = op == kOpFwd ? (int64_t)pb.K * pb.P * pb.Q : (int64_t)pb.C * pb.H * pb.W;
    int64_t &out_bs = op == kOpFwd ? q.y_bs : q.x_bs;
    const int64_t caller_bs = out_bs;
    out_bs = sample;
    float *stage = reinterpret_cast<float *>(static_cast<char *>(ws) + pl.stage_off);
    int rc = run_colgemm_f32out(op, act, w, stage, q, pl, ws, st, ep, &applied);
    if (rc != kStatusOk) return rc;
    if (ep && !applied) {
        rc = run_epilogue_pass(stage, false, sample, *ep, pb.N, rows, plane, st);
        if (rc != kStatusOk) return rc;
    }
    const int64_t count = pb.N * sample;
    hipLaunchKernelGGL(narrow_to_bf16_strided, dim3(grid1d(count, 256)), dim3(256), 0, st, stage,
                       static_cast<unsigned short *>(out), count, sample, caller_bs);
    return check_launch();
}

int run_colgemm_f32out(int op, const void *act, const void *w, void *out, const Problem &caller_pb, const Plan &pl,
                       void *ws, hipStream_t st, const Epilogue *ep, bool *ep_applied)
{
    Problem pb = caller_pb;                     // batch stride of a widened input changes below
    char *wsb = static_cast<char *>(ws);
    int4 *tab = reinterpret_cast<int4 *>(wsb + pl.tab_off);
    float *wt = reinterpret_cast<float *>(wsb + pl.wt_off);
    const int RS = pb.R * pb.S;
    const bool fwd = op == kOpFwd;
    const int Cr = fwd ? pb.C : pb.K;          // channels of the gathered tensor
    const bool fast = Cr % kChunk == 0 && (fwd || pb.stride == 1);
    const bool bf = pb.dtype == kDtypeBf16 && !pl.widen_w;   // bf16 MFMA kernel reads the caller's tensors directly
    int64_t w_bs = (int64_t)pb.K * pb.C * RS;
    if (pl.dma) return run_colgemm_dma(op, act, w, out, pb, pl, ws, st, ep, ep_applied);
    if (pl.patch && pb.dtype == kDtypeBf16) {
        const int rc = run_patch_bf16(act, w, out, pb, pl, ws, st, ep, ep_applied);
        if (rc != kNotTaken) return rc;
    }
    const float *actf = fwd ? as_f32(pl.widen, act, pb.N, (int64_t)pb.C * pb.H * pb.W, &pb.x_bs, wsb, pl, 0, st)
                            : as_f32(pl.widen, act, pb.N, (int64_t)pb.K * pb.P * pb.Q, &pb.y_bs, wsb, pl, 0, st);
    const float *wf = as_f32(pl.widen_w, w, 1, w_bs, &w_bs, wsb, pl, 1, st);

    if (fast) {
        const int kc = bf ? bf16_step_channels(Cr) : pl.kc;
        const int64_t wt_elems = (int64_t)pl.Mpad * Cr * RS;
        const int GF = pl.fused_groups ? pb.groups : 1;      // columns of a grouped layer run in this one launch
        if (bf)
            hipLaunchKernelGGL(relayout_filters_cblk_bf16, dim3(grid1d(wt_elems * GF, 256)), dim3(256), 0, st,
                               static_cast<const unsigned short *>(w), reinterpret_cast<unsigned short *>(wt), pl.M,
                               pl.Mpad, Cr / kc, RS, pb.C, fwd ? 0 : 1, kc, GF, pb.w_gs);
        else if (wt_elems * GF < ((int64_t)1 << 31))
            hipLaunchKernelGGL(relayout_filters_cblk_x4, dim3(grid1d(wt_elems * GF / 4, 256)), dim3(256), 0, st, wf, wt,
                               pl.M, pl.Mpad, Cr / kc, RS, pb.C, fwd ? 0 : 1, kc, GF, pb.w_gs,
                               make_fastdiv((uint32_t)pl.Mpad), make_fastdiv((uint32_t)RS),
                               make_fastdiv((uint32_t)(Cr / kc)));
        else
            hipLaunchKernelGGL(relayout_filters_cblk, dim3(grid1d(wt_elems * GF, 256)), dim3(256), 0, st, wf, wt, pl.M,
                               pl.Mpad, Cr / kc, RS, pb.C, fwd ? 0 : 1, kc, GF, pb.w_gs);
        ColGemmFastArgs a;
        a.At = wt; a.src = actf; a.dst = static_cast<float *>(out);
        a.M = pl.M; a.Mpad = pl.Mpad; a.cblocks = Cr / kc; a.R = pb.R; a.S = pb.S;
        if (fwd) {
            a.sign = 1; a.OH = pb.P; a.OW = pb.Q; a.LH = pb.H; a.LW = pb.W;
            a.src_bs = (int)pb.x_bs; a.dst_bs = (int)pb.y_bs; a.mul = pb.stride; a.add = -pb.pad;
        } else {
            a.sign = -1; a.OH = pb.H; a.OW = pb.W; a.LH = pb.P; a.LW = pb.Q;
            a.src_bs = (int)pb.y_bs; a.dst_bs = (int)pb.x_bs; a.mul = 1; a.add = pb.pad;
        }
        a.plane_bytes = a.LH * a.LW * 4;
        if (bf) {
            // channel-blocked copy of the gathered tensor: 32 bytes per position and block of 16 channels (the
            // columns of a grouped layer are consecutive channel ranges of one tensor: one copy for all of them)
            const int LHW = a.LH * a.LW;
            const int64_t vecs = (int64_t)pb.N * (Cr * GF / 16) * LHW;
            u32x4 *blk = reinterpret_cast<u32x4 *>(wsb + pl.blk_off);
            hipLaunchKernelGGL(block_channels_bf16, dim3(grid1d(vecs, 256)), dim3(256), 0, st,
                               static_cast<const unsigned short *>(act), blk, pb.N, Cr * GF, LHW, (int64_t)a.src_bs,
                               make_fastdiv((uint32_t)LHW));
            a.src = reinterpret_cast<const float *>(blk);
            a.src_bs = (Cr * GF / 16) * LHW;
            a.plane_bytes = LHW * 32;
        }
        a.ncols = pb.N * a.OH * a.OW;
        a.mtiles = pl.Mpad / pl.tile.bm();
        a.ntiles = ceil_div(a.ncols, pl.tile.bn());
        a.div_plane = make_fastdiv((uint32_t)(a.OH * a.OW));
        a.div_ow = make_fastdiv((uint32_t)a.OW);
        a.div_rs = make_fastdiv((uint32_t)RS);
        a.div_s = make_fastdiv((uint32_t)pb.S);
        a.ksplit = pl.nsplit;
        a.out_bf16 = bf && pb.out_bf16;
        a.steps_per_split = ceil_div(a.cblocks * RS, pl.nsplit);      // same ranges as planned, in steps of kc
        a.part = reinterpret_cast<float *>(wsb + pl.part_off);
        a.groups = GF;
        a.src_gs = fwd ? pb.x_gs : pb.y_gs;
        a.dst_gs = fwd ? pb.y_gs : pb.x_gs;
        a.at_gs = wt_elems;
        a.part_gs = (int64_t)(pl.part_bytes / 4);
        a.src_gb = (int64_t)(Cr / 16) * a.LH * a.LW * 32;          // bf16 kernel: channel blocks of one column
        a.at_gb = wt_elems * 2;
        a.dst_gb = a.dst_gs * (a.out_bf16 ? 2 : 4);
        // the 32 x 32 tile kernels and the split-sum kernel apply an epilogue themselves (one column only)
        a.epi_on = ep && GF == 1 && pb.groups == 1 && (bf || pl.tile.mfma != 16 || a.ksplit > 1);
        a.epi = ep ? *ep : Epilogue{};
        *ep_applied = a.epi_on;
        const int need_lds = 2 * (pl.tile.bm() + pl.tile.bn()) * (bf ? kc * 2 + 16 : (kc + 4) * 4);
        const GridPlan g = plan_grid(a.mtiles * a.ntiles * a.ksplit * GF, need_lds);
        a.tiles_per_xcd = g.tiles_per_xcd;
        if (bf) launch_colgemm_bf16(pl.tile, kc, a, g, st);
        else launch_colgemm_fast(pl.tile, kc, a, g, st);
        int rc = check_launch();
        if (rc != kStatusOk || a.ksplit == 1) return rc;
        const int per_sample = a.M * a.OH * a.OW;
        if (a.out_bf16)
            for (int gc = 0; gc < GF; ++gc)
                hipLaunchKernelGGL(reduce_split_outputs<unsigned short>, dim3(2048), dim3(256), 0, st,
                                   a.part + gc * a.part_gs, reinterpret_cast<unsigned short *>(a.dst) + gc * a.dst_gs,
                                   a.ksplit, per_sample, pb.N, a.dst_bs, make_fastdiv((uint32_t)per_sample), a.epi_on,
                                   a.epi, a.div_plane);
        else
            for (int gc = 0; gc < GF; ++gc)
                hipLaunchKernelGGL(reduce_split_outputs<float>, dim3(2048), dim3(256), 0, st, a.part + gc * a.part_gs,
                                   a.dst + gc * a.dst_gs, a.ksplit, per_sample, pb.N, a.dst_bs,
                                   make_fastdiv((uint32_t)per_sample), a.epi_on, a.epi, a.div_plane);
        return check_launch();
    }
    // forward with few channels: the input rows of a tile are staged once in LDS (reads fp32 or bf16 itself and
    // writes the caller's output type)
    if (pl.patch) {
        const int tm = pl.patch_tm, bm = tm * 32, mpad = round_up(pl.M, bm);
        const int PQ = pb.P * pb.Q;
        hipLaunchKernelGGL(relayout_filters, dim3(grid1d((int64_t)mpad * pl.Kgpad, 256)), dim3(256), 0, st, wf, wt,
                           pl.M, mpad, pl.Kg, pl.Kgpad, pb.C, RS, 0);
        PatchArgs a;
        a.At = wt; a.x = act; a.y = out;
        a.M = pl.M; a.Mpad = mpad; a.nchunks = pl.Kgpad / kChunk;
        a.C = pb.C; a.H = pb.H; a.W = pb.W; a.R = pb.R; a.S = pb.S; a.stride = pb.stride; a.pad = pb.pad;
        a.P = pb.P; a.Q = pb.Q; a.PQ = PQ; a.NR = pl.patch_nr; a.WP = pl.patch_wp; a.Kg = pl.Kg; a.Kgpad = pl.Kgpad;
        a.x_bs = (int)pb.x_bs; a.y_bs = (int)pb.y_bs;
        a.mtiles = mpad / bm; a.jtiles = ceil_div(PQ, 128);
        a.ntiles = pb.N * a.mtiles * a.jtiles;
        a.tiles_per_xcd = ceil_div(a.ntiles, 8);
        a.div_q = make_fastdiv((uint32_t)pb.Q);
        a.div_rs = make_fastdiv((uint32_t)RS);
        a.div_s = make_fastdiv((uint32_t)pb.S);
        a.div_mj = make_fastdiv((uint32_t)(a.mtiles * a.jtiles));
        a.div_m = make_fastdiv((uint32_t)a.mtiles);
        a.div_wp = make_fastdiv((uint32_t)pl.patch_wp);
        a.div_nr = make_fastdiv((uint32_t)pl.patch_nr);
        a.div_pr = make_fastdiv((uint32_t)std::max(pb.W / 4, 1));
        a.vec = pb.dtype != kDtypeBf16 && pb.W % 4 == 0 && pb.pad % 2 == 0 && pl.patch_wp % 2 == 0 &&
                pb.x_bs % 4 == 0 && reinterpret_cast<uintptr_t>(act) % 16 == 0;
        // forward only, so an epilogue here is bias / ReLU: applied to the fp32 sums in the kernel's store
        a.epi_on = ep != nullptr;
        a.epi = ep ? *ep : Epilogue{};
        *ep_applied = a.epi_on;
        launch_patch(tm, a, 8 * a.tiles_per_xcd, pl.patch_lds, pb.dtype == kDtypeBf16, pb.out_bf16, st);
        return check_launch();
    }
    if (fwd)
        hipLaunchKernelGGL(build_tap_table, dim3(grid1d(pl.tab_len, 256)), dim3(256), 0, st, tab, pl.tab_len,
                           pl.Kg, RS, pb.S, pb.H * pb.W, pb.W, 1, 1);
    else
        hipLaunchKernelGGL(build_tap_table, dim3(grid1d(pl.tab_len, 256)), dim3(256), 0, st, tab, pl.tab_len,
                           pl.Kg, RS, pb.S, pb.P * pb.Q, pb.stride == 1 ? pb.Q : 0,
                           pb.stride == 1 ? 1 : 0, -1);
    hipLaunchKernelGGL(relayout_filters, dim3(grid1d((int64_t)pl.Mpad * pl.Kgpad, 256)), dim3(256), 0, st, wf, wt,
                       pl.M, pl.Mpad, pl.Kg, pl.Kgpad, pb.C, RS, fwd ? 0 : 1);

    ColGemmArgs a;
    a.At = wt; a.tab = tab; a.src = actf; a.dst = static_cast<float *>(out);
    a.M = pl.M; a.Mpad = pl.Mpad; a.nchunks = pl.Kgpad / kChunk;
    if (fwd) {
        a.OH = pb.P; a.OW = pb.Q; a.LH = pb.H; a.LW = pb.W;
        a.src_bs = (int)pb.x_bs; a.dst_bs = (int)pb.y_bs;
        a.mul = pb.stride; a.add = -pb.pad;
    } else {
        a.OH = pb.H; a.OW = pb.W; a.LH = pb.P; a.LW = pb.Q;
        a.src_bs = (int)pb.y_bs; a.dst_bs = (int)pb.x_bs;
        a.mul = 1; a.add = pb.pad;
    }
    a.ncols = pb.N * a.OH * a.OW;
    a.mtiles = pl.Mpad / pl.tile.bm();
    a.ntiles = ceil_div(a.ncols, pl.tile.bn());
    a.div_plane = make_fastdiv((uint32_t)(a.OH * a.OW));
    a.div_ow = make_fastdiv((uint32_t)a.OW);
    a.div_stride = make_fastdiv((uint32_t)pb.stride);
    const GridPlan g = plan_grid(a.mtiles * a.ntiles, 2 * (pl.tile.bm() + pl.tile.bn()) * kPitch * 4);
    a.tiles_per_xcd = g.tiles_per_xcd;
    if (!fwd && pb.stride > 1) launch_colgemm<kGatherStridedBwd>(pl.tile, a, g, st);
    else launch_colgemm<kGatherDirect>(pl.tile, a, g, st);
    return check_launch();
}

int run_wgrad(const void *x, const void *dy, void *dw, const Problem &caller_pb, const Plan &pl, void *ws,
              hipStream_t st)
{
    Problem pb = caller_pb;                     // batch strides of widened inputs change below
    char *wsb = static_cast<char *>(ws);
    int4 *tab = reinterpret_cast<int4 *>(wsb + pl.tab_off);
    const int RS = pb.R * pb.S;
    // bf16 MFMA kernel: reads the caller's bf16 tensors directly (128-column tiles only)
    const bool bf = pb.dtype == kDtypeBf16 && !pl.widen && pb.C % kChunk == 0;     // bf16 MFMA kernel
    if (pl.lin) {
        // same-extent stride-1 layer: pack both tensors, then every operand is a 16-byte load
        unsigned short *dyp = reinterpret_cast<unsigned short *>(wsb + pl.lin_dy_off);
        unsigned short *xp = reinterpret_cast<unsigned short *>(wsb + pl.lin_x_off);
        const int row_elems = pl.lin_steps * 64;
        PackLinArgs q;
        q.dy = static_cast<const unsigned short *>(dy); q.x = static_cast<const unsigned short *>(x);
        q.dyp = dyp; q.xp = xp;
        q.N = pb.N; q.K = pb.K; q.C = pb.C; q.P = pb.P; q.Q = pb.Q; q.H = pb.H; q.W = pb.W; q.pad = pb.pad;
        q.Wq = pl.lin_wq; q.Jy = pl.lin_jy; q.Jx = pl.lin_jx; q.row_elems = row_elems;
        q.dy_blocks = grid1d((int64_t)pb.K * row_elems / 8, 256);
        q.kpad = round_up(pb.K, 128);
        q.dy_bs = pb.y_bs; q.x_bs = pb.x_bs;
        q.div_row = make_fastdiv((uint32_t)row_elems);
        q.div_jy = make_fastdiv((uint32_t)pl.lin_jy);
        q.div_jx = make_fastdiv((uint32_t)pl.lin_jx);
        q.div_wq = make_fastdiv((uint32_t)pl.lin_wq);
        hipLaunchKernelGGL(pack_lin, dim3(q.dy_blocks + grid1d((int64_t)pb.C * pb.N * pl.lin_jx / 8, 256)), dim3(256),
                           0, st, q);
        WgradLinDmaArgs a;
        a.dyT = dyp; a.xp = xp; a.part = reinterpret_cast<float *>(wsb + pl.part_off);
        a.K = pb.K; a.Kpad = round_up(pb.K, 128); a.C = pb.C; a.ncols = pl.Kg; a.S = pb.S; a.Wq = pl.lin_wq;
        a.N = pb.N; a.G = pl.lin_jy / 8; a.Jx = pl.lin_jx;
        a.row_x_bytes = pb.N * pl.lin_jx * 2;
        a.steps = pl.lin_steps; a.steps_per_split = pl.chunks_per_split;
        a.mtiles = a.Kpad / 128;
        a.ntiles = ceil_div(pl.Kg, 256);
        a.nunits = a.mtiles * a.ntiles * pl.nsplit;
        a.units_per_xcd = ceil_div(a.nunits, 8);
        a.div_c = make_fastdiv((uint32_t)pb.C);
        a.div_s = make_fastdiv((uint32_t)pb.S);
        a.div_g = make_fastdiv((uint32_t)a.G);
        {
            const int lds = 3 * (128 + 256) * 128;
            (void)hipFuncSetAttribute(reinterpret_cast<const void *>(wgrad_bf16_lin_dma_kernel<2, 2, 2, 4>),
                                      hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
            hipLaunchKernelGGL((wgrad_bf16_lin_dma_kernel<2, 2, 2, 4>), dim3(8 * a.units_per_xcd), dim3(512), lds, st, a);
        }
        int rc = check_launch();
        if (rc != kStatusOk) return rc;
        return launch_finish_wgrad(a.part, static_cast<float *>(dw), pb.K, pb.C, RS, pl.nsplit, 1, st);
    }
    if (pl.rows && reinterpret_cast<uintptr_t>(x) % 16 == 0 && reinterpret_cast<uintptr_t>(dy) % 4 == 0) {
        // few channels, stride 4, bf16: input rows as shifted copies in LDS, one partial result per work-group
        WgradRowsArgs a;
        a.x = static_cast<const unsigned short *>(x); a.dy = static_cast<const unsigned short *>(dy);
        a.part = reinterpret_cast<float *>(wsb + pl.part_off);
        a.N = pb.N; a.C = pb.C; a.H = pb.H; a.W = pb.W; a.K = pb.K; a.R = pb.R; a.S = pb.S; a.P = pb.P; a.Q = pb.Q;
        a.Kg = pl.Kg;
        a.x_bs = (int)pb.x_bs; a.y_bs = (int)pb.y_bs;         // N * stride * 4 bytes < 2^31 (problem checks)
        a.dy_elems = (int)((int64_t)(pb.N - 1) * pb.y_bs + (int64_t)pb.K * pb.P * pb.Q);
        a.splits = pl.rows_splits; a.units = pb.N * pl.rows_splits;
        a.ng = ceil_div(pb.Q, 8); a.nkb = ceil_div(pb.Q, 16); a.nnew = pb.R < 4 ? pb.R : 4;
        a.div_splits = make_fastdiv((uint32_t)a.splits);
        a.div_ng = make_fastdiv((uint32_t)a.ng);
        const bool full = pb.S == 11 && a.nkb == 4;             // the first layer: compile-time extents
        const void *kern = full ? reinterpret_cast<const void *>(wgrad_rows_bf16_kernel<true>)
                                : reinterpret_cast<const void *>(wgrad_rows_bf16_kernel<false>);
        if (pl.rows_lds > 64 * 1024)
            (void)hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (full) hipLaunchKernelGGL(wgrad_rows_bf16_kernel<true>, dim3(pl.rows_wgs), dim3(256), pl.rows_lds, st, a);
        else hipLaunchKernelGGL(wgrad_rows_bf16_kernel<false>, dim3(pl.rows_wgs), dim3(256), pl.rows_lds, st, a);
        int rc = check_launch();
        if (rc != kStatusOk) return rc;
        const int count = pb.K * pl.Kg;
        if (count % 4 == 0 && reinterpret_cast<uintptr_t>(dw) % 16 == 0)
            hipLaunchKernelGGL(reduce_partials_x4, dim3(grid1d(count, 64)), dim3(256), 0, st, a.part,
                               static_cast<float *>(dw), count, pl.rows_wgs);
        else
            hipLaunchKernelGGL(reduce_partials, dim3(grid1d(count, 64)), dim3(256), 0, st, a.part,
                               static_cast<float *>(dw), count, pl.rows_wgs);
        return check_launch();
    }
    if (pl.rows_f32) {
        // few channels, fp32: the input rows of an output row in LDS, one partial result per work-group
        WgradRowsF32Args a;
        a.x = static_cast<const float *>(x); a.dy = static_cast<const float *>(dy);
        a.part = reinterpret_cast<float *>(wsb + pl.part_off);
        a.N = pb.N; a.C = pb.C; a.H = pb.H; a.W = pb.W; a.K = pb.K; a.R = pb.R; a.S = pb.S; a.P = pb.P; a.Q = pb.Q;
        a.Kg = pl.Kg; a.stride = pb.stride; a.pad = pb.pad;
        a.x_bs = (int)pb.x_bs; a.y_bs = (int)pb.y_bs;
        a.splits = pl.rows_splits; a.units = pb.N * pl.rows_splits;
        a.WP = pl.rows_wp; a.nnew = pb.R < pb.stride ? pb.R : pb.stride;
        a.div_splits = make_fastdiv((uint32_t)a.splits);
        if (pl.rows_lds > 64 * 1024)
            (void)hipFuncSetAttribute(reinterpret_cast<const void *>(wgrad_rows_f32_kernel),
                                      hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        hipLaunchKernelGGL(wgrad_rows_f32_kernel, dim3(pl.rows_wgs), dim3(kRowsF32Threads), pl.rows_lds, st, a);
        int rc = check_launch();
        if (rc != kStatusOk) return rc;
        const int count = pb.K * pl.Kg;
        if (count % 4 == 0 && reinterpret_cast<uintptr_t>(dw) % 16 == 0)
            hipLaunchKernelGGL(reduce_partials_x4, dim3(grid1d(count, 64)), dim3(256), 0, st, a.part,
                               static_cast<float *>(dw), count, pl.rows_wgs);
        else
            hipLaunchKernelGGL(reduce_partials, dim3(grid1d(count, 64)), dim3(256), 0, st, a.part,
                               static_cast<float *>(dw), count, pl.rows_wgs);
        return check_launch();
    }
    const float *xf = as_f32(pl.widen, x, pb.N, (int64_t)pb.C * pb.H * pb.W, &pb.x_bs, wsb, pl, 0, st);
    const float *dyf = as_f32(pl.widen, dy, pb.N, (int64_t)pb.K * pb.P * pb.Q, &pb.y_bs, wsb, pl, 1, st);
    if (pb.C % kChunk == 0) {
        WgradFastArgs a;
        a.dy = dyf; a.x = xf; a.part = reinterpret_cast<float *>(wsb + pl.part_off);
        a.K = pb.K; a.C = pb.C; a.S = pb.S; a.ncols = pl.Kg;
        a.P = pb.P; a.Q = pb.Q; a.H = pb.H; a.W = pb.W; a.stride = pb.stride; a.pad = pb.pad;
        a.dy_bs = (int)pb.y_bs; a.x_bs = (int)pb.x_bs;
        a.J = pb.N * pb.P * pb.Q;
        a.chunks_per_split = pl.chunks_per_split;
        a.mtiles = pl.Mpad / pl.tile.bm();
        a.ntiles = ceil_div(pl.Kg, pl.tile.bn());
        const int GF = pl.fused_groups ? pb.groups : 1;      // columns of a grouped layer run in this one launch
        a.nsplit = pl.nsplit; a.groups = GF;
        a.dy_gs = pb.y_gs; a.x_gs = pb.x_gs; a.part_gs = (int64_t)(pl.part_bytes / 4);
        a.nunits = a.mtiles * a.ntiles * pl.nsplit * GF;
        const int need_lds = 2 * (pl.tile.bm() + pl.tile.bn()) * (bf ? kWgradBf16Depth * 2 + 16 : kPitch * 4);
        const GridPlan g = plan_grid(a.nunits, need_lds);
        a.units_per_xcd = g.tiles_per_xcd;
        a.x_plane_bytes = pb.H * pb.W * (bf ? 2 : 4);
        a.y_plane_bytes = pb.P * pb.Q * (bf ? 2 : 4);
        a.div_plane = make_fastdiv((uint32_t)(pb.P * pb.Q));
        a.div_q = make_fastdiv((uint32_t)pb.Q);
        a.div_c = make_fastdiv((uint32_t)pb.C);
        if (bf) launch_wgrad_bf16(pl.tile, a, g.grid, need_lds + g.dyn_lds, st);
        else launch_wgrad_fast(pl.tile, a, g, st);
        int rc = check_launch();
        if (rc != kStatusOk) return rc;
        return launch_finish_wgrad(a.part, static_cast<float *>(dw), pb.K, pb.C, RS, pl.nsplit, GF, st);
    }
    hipLaunchKernelGGL(build_tap_table, dim3(grid1d(pl.tab_len, 256)), dim3(256), 0, st, tab, pl.tab_len, pl.Kg, RS,
                       pb.S, pb.H * pb.W, pb.W, 1, 1);
    WgradArgs a;
    a.dy = dyf; a.x = xf; a.tab = tab;
    a.out = pl.nsplit > 1 ? reinterpret_cast<float *>(wsb + pl.part_off) : static_cast<float *>(dw);
    a.K = pb.K; a.CRS = pl.Kg;
    a.P = pb.P; a.Q = pb.Q; a.H = pb.H; a.W = pb.W; a.stride = pb.stride; a.pad = pb.pad;
    a.dy_bs = (int)pb.y_bs; a.x_bs = (int)pb.x_bs;
    a.J = pb.N * pb.P * pb.Q;
    a.chunks_per_split = pl.chunks_per_split;
    a.mtiles = pl.Mpad / pl.tile.bm();
    a.ntiles = ceil_div(pl.Kg, pl.tile.bn());
    a.div_plane = make_fastdiv((uint32_t)(pb.P * pb.Q));
    a.div_q = make_fastdiv((uint32_t)pb.Q);
    // the table kernel reads fp32 or bf16 inputs itself
    a.units = a.mtiles * a.ntiles * pl.nsplit;
    a.units_per_xcd = ceil_div(a.units, 8);
    launch_wgrad(pl.tile, a, 8 * a.units_per_xcd, pb.dtype == kDtypeBf16, st);
    int rc = check_launch();
    if (rc != kStatusOk) return rc;
    if (pl.nsplit > 1) {
        const int count = pb.K * pl.Kg;
        hipLaunchKernelGGL(reduce_partials, dim3(grid1d(count, 64)), dim3(256), 0, st, a.out,
                           static_cast<float *>(dw), count, pl.nsplit);
        rc = check_launch();
    }
    return rc;
}

int pool_checks(int64_t planes, int H, int W, int &PH, int &PW)
{
    if (planes <= 0 || H < 3 || W < 3) return kErrInvalidArg;
    PH = (H - 3) / 2 + 1;
    PW = (W - 3) / 2 + 1;
    if ((double)planes * H * W * 4.0 >= (double)((int64_t)1 << 40) || (int64_t)H * W >= (1 << 30)) return kErrTooLarge;
    return kStatusOk;
}

// element type of the glue tensors: fp32 for kDtypeF32, bfloat16 for the two bf16 codes
int glue_elem_bytes(int dtype)
{
    if (dtype == kDtypeF32) return 4;
    if (dtype == kDtypeBf16 || dtype == kDtypeBf16OutBf16) return 2;
    return 0;
}

// window rows of loads a lane of the walking pooling kernels keeps in flight (4: best of 3, 4 and 6 as measured)
constexpr int kPoolWalkDepth = 4;

template <bool RELU, typename T>
int pool_fwd_typed(const void *x, void *y, int64_t planes, int H, int W, int PH, int PW, hipStream_t st)
{
    if (PW + 1 <= 64) {                          // a plane's column pairs fit a wavefront: walk down the planes
        const int seg = PW + 1, ppw = 64 / seg;
        const int64_t waves = (planes + ppw - 1) / ppw;
        hipLaunchKernelGGL((maxpool_fwd_walk<RELU, T, kPoolWalkDepth>), dim3((unsigned)((waves + 3) / 4)), dim3(256),
                           0, st, static_cast<const T *>(x), static_cast<T *>(y), planes, H, W, PH, PW, seg, ppw,
                           make_fastdiv((uint32_t)seg));
        return check_launch();
    }
    const int64_t total = planes * PH * PW;
    hipLaunchKernelGGL((maxpool_fwd_kernel<RELU, T>), dim3(grid1d(total, 256)), dim3(256), 0, st,
                       static_cast<const T *>(x), static_cast<T *>(y), total, H, W, PH, PW,
                       make_fastdiv((uint32_t)PW), make_fastdiv((uint32_t)PH));
    return check_launch();
}

template <bool RELU>
int pool_fwd_impl(const void *x, void *y, int64_t planes, int H, int W, int dtype, void *stream)
{
    if (!x || !y) return kErrInvalidArg;
    int PH, PW;
    int rc = pool_checks(planes, H, W, PH, PW);
    if (rc != kStatusOk) return rc;
    const int eb = glue_elem_bytes(dtype);
    if (!eb) return kErrBadDtype;
    if (!aligned(x, eb) || !aligned(y, eb)) return kErrMisaligned;
    hipStream_t st = static_cast<hipStream_t>(stream);
    return eb == 4 ? pool_fwd_typed<RELU, float>(x, y, planes, H, W, PH, PW, st)
                   : pool_fwd_typed<RELU, unsigned short>(x, y, planes, H, W, PH, PW, st);
}

template <bool RELU, typename T>
int pool_bwd_typed(const void *x, const void *dy, void *dx, int64_t planes, int H, int W, int PH, int PW,
                   hipStream_t st)
{
    const T *xp = static_cast<const T *>(x), *gp = static_cast<const T *>(dy);
    T *op = static_cast<T *>(dx);
    if (PW + 1 <= 64) {                          // a plane's column pairs fit a wavefront: walk down the planes
        const int seg = PW + 1, ppw = 64 / seg;
        const int64_t waves = (planes + ppw - 1) / ppw;
        hipLaunchKernelGGL((maxpool_bwd_walk<RELU, T, kPoolWalkDepth>), dim3((unsigned)((waves + 3) / 4)), dim3(256),
                           0, st, xp, gp, op, planes, H, W, PH, PW, seg, ppw, make_fastdiv((uint32_t)seg));
    } else {
        const int64_t total = planes * H * W;
        hipLaunchKernelGGL((maxpool_bwd_kernel<RELU, T>), dim3(grid1d(total, 256)), dim3(256), 0, st, xp, gp, op,
                           total, H, W, PH, PW);
    }
    return check_launch();
}

template <bool RELU>
int pool_bwd_impl(const void *x, const void *dy, void *dx, int64_t planes, int H, int W, int dtype, void *stream)
{
    if (!x || !dy || !dx) return kErrInvalidArg;
    int PH, PW;
    int rc = pool_checks(planes, H, W, PH, PW);
    if (rc != kStatusOk) return rc;
    const int eb = glue_elem_bytes(dtype);
    if (!eb) return kErrBadDtype;
    if (!aligned(x, eb) || !aligned(dy, eb) || !aligned(dx, eb)) return kErrMisaligned;
    hipStream_t st = static_cast<hipStream_t>(stream);
    return eb == 4 ? pool_bwd_typed<RELU, float>(x, dy, dx, planes, H, W, PH, PW, st)
                   : pool_bwd_typed<RELU, unsigned short>(x, dy, dx, planes, H, W, PH, PW, st);
}

template <typename T>
int relu_fwd_typed(const void *x, void *y, int64_t count, hipStream_t st)
{
    constexpr int V = 16 / (int)sizeof(T);
    const int vec = aligned(x, 16) && aligned(y, 16);
    const int64_t threads = vec ? count / V + V : count;
    hipLaunchKernelGGL(relu_fwd_kernel<T>, dim3(grid1d(threads, 256)), dim3(256), 0, st, static_cast<const T *>(x),
                       static_cast<T *>(y), count, vec);
    return check_launch();
}

template <typename T>
int relu_bwd_typed(const void *x, const void *dy, void *dx, int64_t count, hipStream_t st)
{
    constexpr int V = 16 / (int)sizeof(T);
    const int vec = aligned(x, 16) && aligned(dy, 16) && aligned(dx, 16);
    const int64_t threads = vec ? count / V + V : count;
    hipLaunchKernelGGL(relu_bwd_kernel<T>, dim3(grid1d(threads, 256)), dim3(256), 0, st, static_cast<const T *>(x),
                       static_cast<const T *>(dy), static_cast<T *>(dx), count, vec);
    return check_launch();
}

}  // namespace

extern "C" {

int conv_fwd_ex(const void *x, const void *w, void *y, int N, int C, int H, int W, int K, int R, int S, int stride,
                int pad, int64_t x_batch_stride, int64_t y_batch_stride, int dtype, void *ws, size_t ws_bytes,
                void *stream)
{
    Problem pb; Plan pl;
    int rc = prepare(kOpFwd, x, w, y, N, C, H, W, K, R, S, stride, pad, x_batch_stride, y_batch_stride, dtype, ws,
                     ws_bytes, pb, pl);
    if (rc != kStatusOk) return rc;
    return run_colgemm(kOpFwd, x, w, y, pb, pl, ws, static_cast<hipStream_t>(stream));
}

int conv_bwd_data_ex(const void *dy, const void *w, void *dx, int N, int C, int H, int W, int K, int R, int S,
                     int stride, int pad, int64_t x_batch_stride, int64_t y_batch_stride, int dtype, void *ws,
                     size_t ws_bytes, void *stream)
{
    Problem pb; Plan pl;
    int rc = prepare(kOpBwdData, dy, w, dx, N, C, H, W, K, R, S, stride, pad, x_batch_stride, y_batch_stride, dtype,
                     ws, ws_bytes, pb, pl);
    if (rc != kStatusOk) return rc;
    return run_colgemm(kOpBwdData, dy, w, dx, pb, pl, ws, static_cast<hipStream_t>(stream));
}

int conv_fwd_bias_relu(const void *x, const void *w, const void *bias, void *y, int N, int C, int H, int W, int K,
                       int R, int S, int stride, int pad, int relu, int dtype, void *ws, size_t ws_bytes, void *stream)
{
    if (relu != 0 && relu != 1) return kErrInvalidArg;
    if (bias && !aligned(bias, 4)) return kErrMisaligned;
    Problem pb; Plan pl;
    int rc = prepare(kOpFwd, x, w, y, N, C, H, W, K, R, S, stride, pad, 0, 0, dtype, ws, ws_bytes, pb, pl);
    if (rc != kStatusOk) return rc;
    Epilogue e{};
    e.bias = static_cast<const float *>(bias);
    e.relu = relu;
    const bool any = bias || relu;
    return run_colgemm(kOpFwd, x, w, y, pb, pl, ws, static_cast<hipStream_t>(stream), any ? &e : nullptr);
}

int conv_bwd_data_relu(const void *dy, const void *w, const void *act, void *dx, int N, int C, int H, int W, int K,
                       int R, int S, int stride, int pad, int dtype, void *ws, size_t ws_bytes, void *stream)
{
    if (!act) return kErrInvalidArg;
    if (!aligned(act, 4)) return kErrMisaligned;
    Problem pb; Plan pl;
    int rc = prepare(kOpBwdData, dy, w, dx, N, C, H, W, K, R, S, stride, pad, 0, 0, dtype, ws, ws_bytes, pb, pl);
    if (rc != kStatusOk) return rc;
    Epilogue e{};
    e.mask = act;
    e.mask_bs = pb.x_bs;
    e.mask_bf16 = pb.out_bf16;
    return run_colgemm(kOpBwdData, dy, w, dx, pb, pl, ws, static_cast<hipStream_t>(stream), &e);
}

int conv_bwd_filter_ex(const void *x, const void *dy, void *dw, int N, int C, int H, int W, int K, int R, int S,
                       int stride, int pad, int64_t x_batch_stride, int64_t y_batch_stride, int dtype, void *ws,
                       size_t ws_bytes, void *stream)
{
    Problem pb; Plan pl;
    int rc = prepare(kOpBwdFilter, x, dy, dw, N, C, H, W, K, R, S, stride, pad, x_batch_stride, y_batch_stride,
                     dtype, ws, ws_bytes, pb, pl);
    if (rc != kStatusOk) return rc;
    return run_wgrad(x, dy, dw, pb, pl, ws, static_cast<hipStream_t>(stream));
}

// Grouped layers.  The per-column problem carries the full tensors' batch strides and the column strides; columns
// run in one launch where the plan says so, else one after the other on offset pointers.
static int grouped_problem(Problem &pb, int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                           int groups, int dtype)
{
    if (groups < 1 || C <= 0 || K <= 0 || C % groups != 0 || K % groups != 0) return kErrInvalidArg;
    const int Cg = C / groups, Kg = K / groups;
    int rc = make_problem(pb, N, Cg, H, W, Kg, R, S, stride, pad, 0, 0, dtype);
    if (rc != kStatusOk) return rc;
    // the same checks on the full tensors' spans (the kernels index them with 32-bit byte offsets)
    Problem full;
    rc = make_problem(full, N, C, H, W, K, R, S, stride, pad, 0, 0, dtype);
    if (rc != kStatusOk && rc != kErrTooLarge) return rc;
    if ((int64_t)N * C * H * W * 4 >= kMaxSpanBytes || (int64_t)N * K * pb.P * pb.Q * 4 >= kMaxSpanBytes)
        return kErrTooLarge;
    pb.x_bs = (int64_t)C * H * W;
    pb.y_bs = (int64_t)K * pb.P * pb.Q;
    pb.groups = groups;
    pb.x_gs = (int64_t)Cg * H * W;
    pb.y_gs = (int64_t)Kg * pb.P * pb.Q;
    pb.w_gs = (int64_t)Kg * Cg * R * S;
    return kStatusOk;
}

static int run_grouped(int op, const void *a, const void *b, void *out, int N, int C, int H, int W, int K, int R,
                       int S, int stride, int pad, int groups, int dtype, void *ws, size_t ws_bytes, void *stream)
{
    if (!a || !b || !out) return kErrInvalidArg;
    Problem pb;
    int rc = grouped_problem(pb, N, C, H, W, K, R, S, stride, pad, groups, dtype);
    if (rc != kStatusOk) return rc;
    if (!aligned(a, 16) || !aligned(b, 16) || !aligned(out, 16)) return kErrMisaligned;
    const Plan pl = make_plan(op, pb);
    if (pl.total > 0) {
        if (!ws || ws_bytes < pl.total) return kErrWorkspace;
        if (!aligned(ws, 256)) return kErrMisaligned;
    }
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (groups == 1 || pl.fused_groups)
        return op == kOpBwdFilter ? run_wgrad(a, b, out, pb, pl, ws, st) : run_colgemm(op, a, b, out, pb, pl, ws, st);
    // one column after the other: element sizes of the three tensors of this pass
    const int in_b = pb.dtype == kDtypeBf16 ? 2 : 4;
    const int out_b = (pb.out_bf16 && op != kOpBwdFilter) ? 2 : 4;
    Problem one = pb;
    one.groups = 1;
    // byte distance between the columns' slices of the three tensors
    int64_t sa, sb, so;
    if (op == kOpFwd) { sa = pb.x_gs * in_b; sb = pb.w_gs * in_b; so = pb.y_gs * out_b; }
    else if (op == kOpBwdData) { sa = pb.y_gs * in_b; sb = pb.w_gs * in_b; so = pb.x_gs * out_b; }
    else { sa = pb.x_gs * in_b; sb = pb.y_gs * in_b; so = pb.w_gs * 4; }
    // every column's base must keep the alignment the kernels rely on: checked for all columns before the first
    // one is enqueued
    for (int g = 1; g < groups; ++g)
        if ((g * sa) % 16 != 0 || (g * sb) % 16 != 0 || (g * so) % 16 != 0) return kErrMisaligned;
    for (int g = 0; g < groups; ++g) {
        const char *pa = static_cast<const char *>(a) + g * sa, *pbp = static_cast<const char *>(b) + g * sb;
        char *po = static_cast<char *>(out) + g * so;
        rc = op == kOpBwdFilter ? run_wgrad(pa, pbp, po, one, pl, ws, st) : run_colgemm(op, pa, pbp, po, one, pl, ws, st);
        if (rc != kStatusOk) return rc;
    }
    return kStatusOk;
}

int conv_fwd_grouped(const void *x, const void *w, void *y, int N, int C, int H, int W, int K, int R, int S,
                     int stride, int pad, int groups, int dtype, void *ws, size_t ws_bytes, void *stream)
{
    return run_grouped(kOpFwd, x, w, y, N, C, H, W, K, R, S, stride, pad, groups, dtype, ws, ws_bytes, stream);
}

int conv_bwd_data_grouped(const void *dy, const void *w, void *dx, int N, int C, int H, int W, int K, int R, int S,
                          int stride, int pad, int groups, int dtype, void *ws, size_t ws_bytes, void *stream)
{
    return run_grouped(kOpBwdData, dy, w, dx, N, C, H, W, K, R, S, stride, pad, groups, dtype, ws, ws_bytes, stream);
}

int conv_bwd_filter_grouped(const void *x, const void *dy, void *dw, int N, int C, int H, int W, int K, int R, int S,
                            int stride, int pad, int groups, int dtype, void *ws, size_t ws_bytes, void *stream)
{
    return run_grouped(kOpBwdFilter, x, dy, dw, N, C, H, W, K, R, S, stride, pad, groups, dtype, ws, ws_bytes,
                       stream);
}

size_t conv_workspace_bytes_grouped(int op, int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                                    int groups, int dtype)
{
    if (op != kOpFwd && op != kOpBwdData && op != kOpBwdFilter) return 0;
    Problem pb;
    if (grouped_problem(pb, N, C, H, W, K, R, S, stride, pad, groups, dtype) != kStatusOk) return 0;
    return make_plan(op, pb).total;
}

int conv_fwd(const void *x, const void *w, void *y, int N, int C, int H, int W, int K, int R, int S, int stride,
             int pad, int dtype, void *ws, size_t ws_bytes, void *stream)
{
    return conv_fwd_ex(x, w, y, N, C, H, W, K, R, S, stride, pad, 0, 0, dtype, ws, ws_bytes, stream);
}

int conv_bwd_data(const void *dy, const void *w, void *dx, int N, int C, int H, int W, int K, int R, int S,
                  int stride, int pad, int dtype, void *ws, size_t ws_bytes, void *stream)
{
    return conv_bwd_data_ex(dy, w, dx, N, C, H, W, K, R, S, stride, pad, 0, 0, dtype, ws, ws_bytes, stream);
}

int conv_bwd_filter(const void *x, const void *dy, void *dw, int N, int C, int H, int W, int K, int R, int S,
                    int stride, int pad, int dtype, void *ws, size_t ws_bytes, void *stream)
{
    return conv_bwd_filter_ex(x, dy, dw, N, C, H, W, K, R, S, stride, pad, 0, 0, dtype, ws, ws_bytes, stream);
}

size_t conv_workspace_bytes(int op, int N, int C, int H, int W, int K, int R, int S, int stride, int pad, int dtype)
{
    if (op != kOpFwd && op != kOpBwdData && op != kOpBwdFilter) return 0;
    Problem pb;
    if (make_problem(pb, N, C, H, W, K, R, S, stride, pad, 0, 0, dtype) != kStatusOk) return 0;
    return make_plan(op, pb).total;
}

// Address of this GPU's copy of `scratch`, resolved once per device with that device current.
static int noalloc_scratch(void **out)
{
    constexpr int kMaxDevices = 64;
    static void *ptrs[kMaxDevices] = {};
    static std::mutex mu;
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e);
    if (dev < 0 || dev >= kMaxDevices) return hip_fail(hipErrorInvalidDevice);
    std::lock_guard<std::mutex> lock(mu);
    if (!ptrs[dev]) {
        void *ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return hip_fail(e);
        if (!ptr || !aligned(ptr, 256)) return hip_fail(hipErrorInvalidSymbol);
        ptrs[dev] = ptr;
    }
    *out = ptrs[dev];
    return kStatusOk;
}

int conv_bwd_filter_noalloc(const void *x, const void *dy, void *dw, int N, int C, int H, int W, int K, int R, int S,
                            int stride, int pad, int dtype, void *stream)
{
    if (!x || !dy || !dw) return kErrInvalidArg;
    Problem pb;
    int rc = make_problem(pb, N, C, H, W, K, R, S, stride, pad, 0, 0, dtype);
    if (rc != kStatusOk) return rc;
    if (!aligned(x, 16) || !aligned(dy, 16) || !aligned(dw, 16)) return kErrMisaligned;
    const Plan pl = make_plan(kOpBwdFilter, pb);
    if (pl.total > (size_t)CONV_NOALLOC_SCRATCH_BYTES) return kErrScratchLimit;
    void *ws = nullptr;
    rc = noalloc_scratch(&ws);
    if (rc != kStatusOk) return rc;
    return run_wgrad(x, dy, dw, pb, pl, ws, static_cast<hipStream_t>(stream));
}

int conv_output_extent(int in, int filt, int stride, int pad)
{
    if (in <= 0 || filt <= 0 || stride <= 0 || pad < 0 || pad > (1 << 20)) return 0;
    return out_extent(in, filt, stride, pad);
}

const char *conv_status_string(int status)
{
    switch (status) {
    case kStatusOk: return "ok";
    case kErrInvalidArg: return "invalid argument (null pointer, non-positive extent or empty output)";
    case kErrTooLarge: return "tensor too large (a span reaches 2^31 bytes)";
    case kErrBadDtype: return "unknown dtype";
    case kErrWorkspace: return "workspace missing or too small";
    case kErrMisaligned: return "pointer not sufficiently aligned";
    case kErrHip: return "HIP runtime error";
    case kErrScratchLimit: return "the pass needs more scratch than the library's built-in buffer holds";
    default: return "unknown status";
    }
}

const char *conv_last_hip_error(void) { return g_hip_error; }

int convert_f32_to_bf16(const void *src, void *dst, int64_t count, void *stream)
{
    if (!src || !dst || count < 0) return kErrInvalidArg;
    if (count == 0) return kStatusOk;
    if (!aligned(src, 4) || !aligned(dst, 2)) return kErrMisaligned;
    hipLaunchKernelGGL(narrow_to_bf16, dim3(grid1d(count, 256)), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const float *>(src), static_cast<unsigned short *>(dst), count);
    return check_launch();
}

// samples per filter are spread over this many work-groups in the bias gradient (about 2048 work-groups)
static int bias_splits(int N, int K)
{
    int s = 2048 / K;
    if (s < 1) s = 1;
    return s < N ? s : N;
}

size_t bias_bwd_workspace_bytes(int N, int K)
{
    if (N <= 0 || K <= 0) return 0;
    return (size_t)K * bias_splits(N, K) * 4;
}

int bias_fwd(void *y, const void *b, int N, int K, int PQ, int dtype, void *stream)
{
    if (!y || !b || N <= 0 || K <= 0 || PQ <= 0) return kErrInvalidArg;
    const int eb = glue_elem_bytes(dtype);
    if (!eb) return kErrBadDtype;
    const int64_t total = (int64_t)N * K * PQ;
    if (total >= ((int64_t)1 << 31)) return kErrTooLarge;
    if (!aligned(y, eb) || !aligned(b, 4)) return kErrMisaligned;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const FastDiv dpq = make_fastdiv((uint32_t)PQ), dk = make_fastdiv((uint32_t)K);
    if (eb == 4)
        hipLaunchKernelGGL(bias_fwd_kernel<float>, dim3(grid1d(total, 256)), dim3(256), 0, st, static_cast<float *>(y),
                           static_cast<const float *>(b), total, K, dpq, dk);
    else
        hipLaunchKernelGGL(bias_fwd_kernel<unsigned short>, dim3(grid1d(total, 256)), dim3(256), 0, st,
                           static_cast<unsigned short *>(y), static_cast<const float *>(b), total, K, dpq, dk);
    return check_launch();
}

int bias_bwd(const void *dy, void *db, int N, int K, int PQ, int dtype, void *ws, size_t ws_bytes, void *stream)
{
    if (!dy || !db || N <= 0 || K <= 0 || PQ <= 0) return kErrInvalidArg;
    const int eb = glue_elem_bytes(dtype);
    if (!eb) return kErrBadDtype;
    if ((int64_t)N * K * PQ >= ((int64_t)1 << 31)) return kErrTooLarge;
    if (!aligned(dy, eb) || !aligned(db, 4)) return kErrMisaligned;
    if (!ws || ws_bytes < bias_bwd_workspace_bytes(N, K)) return kErrWorkspace;
    if (!aligned(ws, 256)) return kErrMisaligned;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (PQ == 1) {
        if (eb == 4)
            hipLaunchKernelGGL(bias_bwd_columns<float>, dim3(grid1d(K, 64)), dim3(64), 0, st,
                               static_cast<const float *>(dy), static_cast<float *>(db), N, K);
        else
            hipLaunchKernelGGL(bias_bwd_columns<unsigned short>, dim3(grid1d(K, 64)), dim3(64), 0, st,
                               static_cast<const unsigned short *>(dy), static_cast<float *>(db), N, K);
        return check_launch();
    }
    const int nsplit = bias_splits(N, K);
    float *part = static_cast<float *>(ws);
    if (eb == 4)
        hipLaunchKernelGGL(bias_bwd_partial<float>, dim3(K, nsplit), dim3(256), 0, st, static_cast<const float *>(dy),
                           part, N, K, PQ, nsplit);
    else
        hipLaunchKernelGGL(bias_bwd_partial<unsigned short>, dim3(K, nsplit), dim3(256), 0, st,
                           static_cast<const unsigned short *>(dy), part, N, K, PQ, nsplit);
    hipLaunchKernelGGL(bias_bwd_finish, dim3(grid1d(K, 256)), dim3(256), 0, st, part, static_cast<float *>(db), K,
                       nsplit);
    return check_launch();
}

int relu_fwd(const void *x, void *y, int64_t count, int dtype, void *stream)
{
    if (!x || !y || count < 0) return kErrInvalidArg;
    const int eb = glue_elem_bytes(dtype);
    if (!eb) return kErrBadDtype;
    if (count == 0) return kStatusOk;
    if (!aligned(x, eb) || !aligned(y, eb)) return kErrMisaligned;
    hipStream_t st = static_cast<hipStream_t>(stream);
    return eb == 4 ? relu_fwd_typed<float>(x, y, count, st) : relu_fwd_typed<unsigned short>(x, y, count, st);
}

int relu_bwd(const void *x, const void *dy, void *dx, int64_t count, int dtype, void *stream)
{
    if (!x || !dy || !dx || count < 0) return kErrInvalidArg;
    const int eb = glue_elem_bytes(dtype);
    if (!eb) return kErrBadDtype;
    if (count == 0) return kStatusOk;
    if (!aligned(x, eb) || !aligned(dy, eb) || !aligned(dx, eb)) return kErrMisaligned;
    hipStream_t st = static_cast<hipStream_t>(stream);
    return eb == 4 ? relu_bwd_typed<float>(x, dy, dx, count, st)
                   : relu_bwd_typed<unsigned short>(x, dy, dx, count, st);
}

int maxpool3x3s2_fwd(const void *x, void *y, int64_t planes, int H, int W, int dtype, void *stream)
{
    return pool_fwd_impl<false>(x, y, planes, H, W, dtype, stream);
}

int maxpool3x3s2_bwd(const void *x, const void *dy, void *dx, int64_t planes, int H, int W, int dtype, void *stream)
{
    return pool_bwd_impl<false>(x, dy, dx, planes, H, W, dtype, stream);
}

int relu_maxpool3x3s2_fwd(const void *x, void *y, int64_t planes, int H, int W, int dtype, void *stream)
{
    return pool_fwd_impl<true>(x, y, planes, H, W, dtype, stream);
}

int relu_maxpool3x3s2_bwd(const void *x, const void *dy, void *dx, int64_t planes, int H, int W, int dtype,
                          void *stream)
{
    return pool_bwd_impl<true>(x, dy, dx, planes, H, W, dtype, stream);
}

static int run_fc(int op, const void *a, const void *b, void *out, const void *bias, int relu, int N, int I, int O,
                  int dtype, void *ws, size_t ws_bytes, void *stream)
{
    if (!a || !b || !out) return kErrInvalidArg;
    if (relu != 0 && relu != 1) return kErrInvalidArg;
    FcPlan pl;
    int rc = make_fc_plan(pl, op, N, I, O, dtype);
    if (rc != kStatusOk) return rc;
    if (!aligned(a, 16) || !aligned(b, 16) || !aligned(out, 16) || !aligned(bias, 4)) return kErrMisaligned;
    if (pl.part_bytes > 0) {
        if (!ws || ws_bytes < pl.part_bytes) return kErrWorkspace;
        if (!aligned(ws, 256)) return kErrMisaligned;
    }
    hipStream_t st = static_cast<hipStream_t>(stream);
    FcArgs g;
    g.A = static_cast<const float *>(a); g.B = static_cast<const float *>(b);
    g.D = static_cast<float *>(out); g.part = static_cast<float *>(ws);
    g.M = pl.M; g.Nc = pl.Nc; g.K = pl.K; g.lda = pl.lda; g.ldb = pl.ldb; g.ldd = pl.ldd;
    g.mtiles = pl.mtiles; g.ntiles = pl.ntiles; g.ksplit = pl.ksplit; g.steps_per_split = pl.steps_per_split;
    g.bias = static_cast<const float *>(bias); g.relu = relu;
    const dim3 grid(pl.mtiles * pl.ntiles * pl.ksplit), block(kThreads);
    if (pl.at) hipLaunchKernelGGL((fc_gemm_kernel<true, true>), grid, block, 0, st, g);
    else if (pl.bt) hipLaunchKernelGGL((fc_gemm_kernel<false, true>), grid, block, 0, st, g);
    else hipLaunchKernelGGL((fc_gemm_kernel<false, false>), grid, block, 0, st, g);
    rc = check_launch();
    if (rc != kStatusOk || pl.ksplit == 1) return rc;
    hipLaunchKernelGGL(fc_reduce_kernel, dim3(std::min<int64_t>(2048, ((int64_t)pl.M * pl.Nc + 255) / 256)), dim3(256),
                       0, st, g.part, g.D, pl.ksplit, pl.M, pl.Nc, pl.ldd, g.bias, relu);
    return check_launch();
}

int fc_fwd(const void *x, const void *w, const void *bias, void *y, int N, int I, int O, int relu, int dtype,
           void *ws, size_t ws_bytes, void *stream)
{
    return run_fc(kOpFwd, x, w, y, bias, relu, N, I, O, dtype, ws, ws_bytes, stream);
}

int fc_bwd_data(const void *dy, const void *w, void *dx, int N, int I, int O, int dtype, void *ws, size_t ws_bytes,
                void *stream)
{
    return run_fc(kOpBwdData, dy, w, dx, nullptr, 0, N, I, O, dtype, ws, ws_bytes, stream);
}

int fc_bwd_filter(const void *x, const void *dy, void *dw, int N, int I, int O, int dtype, void *ws, size_t ws_bytes,
                  void *stream)
{
    return run_fc(kOpBwdFilter, dy, x, dw, nullptr, 0, N, I, O, dtype, ws, ws_bytes, stream);
}

size_t fc_workspace_bytes(int op, int N, int I, int O, int dtype)
{
    FcPlan pl;
    if (make_fc_plan(pl, op, N, I, O, dtype) != kStatusOk) return 0;
    return pl.part_bytes;
}

int sgd_update(void *w, const void *dw, void *vel, int64_t count, float lr, float momentum, float weight_decay,
               float grad_scale, void *stream)
{
    if (count < 0 || (count > 0 && (!w || !dw || !vel))) return kErrInvalidArg;
    if (count == 0) return kStatusOk;
    if (!aligned(w, 4) || !aligned(dw, 4) || !aligned(vel, 4)) return kErrMisaligned;
    const int vec = aligned(w, 16) && aligned(dw, 16) && aligned(vel, 16);
    const int64_t threads = vec ? std::max<int64_t>((count >> 2), 4) : count;
    if ((threads + 255) / 256 >= ((int64_t)1 << 31)) return kErrTooLarge;
    hipLaunchKernelGGL(sgd_update_kernel, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0,
                       static_cast<hipStream_t>(stream), static_cast<float *>(w), static_cast<const float *>(dw),
                       static_cast<float *>(vel), count, lr, momentum, weight_decay, grad_scale, vec);
    return check_launch();
}

int sgd_update_multi(void *const *w, const void *const *dw, void *const *vel, const int64_t *counts, int ntensors,
                     float lr, float momentum, float weight_decay, float grad_scale, void *stream)
{
    if (ntensors < 0 || (ntensors > 0 && (!w || !dw || !vel || !counts))) return kErrInvalidArg;
    for (int t = 0; t < ntensors; ++t) {
        if (counts[t] < 0 || (counts[t] > 0 && (!w[t] || !dw[t] || !vel[t]))) return kErrInvalidArg;
        if (counts[t] > 0 && (!aligned(w[t], 4) || !aligned(dw[t], 4) || !aligned(vel[t], 4))) return kErrMisaligned;
    }
    // launches of up to kSgdMaxTensors tensors each; tensors without parameters take no blocks
    int t = 0;
    while (t < ntensors) {
        SgdMultiArgs a = {};
        a.lr = lr; a.momentum = momentum; a.weight_decay = weight_decay; a.grad_scale = grad_scale;
        int64_t blocks = 0;
        while (t < ntensors && a.n < kSgdMaxTensors) {
            if (counts[t] > 0) {
                const int vec = aligned(w[t], 16) && aligned(dw[t], 16) && aligned(vel[t], 16);
                const int64_t threads = vec ? std::max<int64_t>(counts[t] >> 2, 4) : counts[t];
                const int64_t nb = (threads + 255) / 256;
                if (blocks + nb >= ((int64_t)1 << 31)) {
                    if (a.n == 0) return kErrTooLarge;
                    break;                                  // this tensor starts the next launch
                }
                a.w[a.n] = static_cast<float *>(w[t]); a.dw[a.n] = static_cast<const float *>(dw[t]);
                a.vel[a.n] = static_cast<float *>(vel[t]); a.count[a.n] = counts[t]; a.vec[a.n] = vec;
                a.first_block[a.n] = (unsigned)blocks;
                blocks += nb;
                ++a.n;
                a.first_block[a.n] = (unsigned)blocks;
            }
            ++t;
        }
        if (a.n == 0) continue;
        hipLaunchKernelGGL(sgd_update_multi_kernel, dim3((unsigned)blocks), dim3(256), 0,
                           static_cast<hipStream_t>(stream), a);
        const int rc = check_launch();
        if (rc != kStatusOk) return rc;
    }
    return kStatusOk;
}

}  // extern "C"
