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
#include <type_traits>
#include <stdlib.h>
#include <string.h>

#include "../../include/convnet_hotpath.h"
#include "plan.h"

using namespace convnet;

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

namespace {

constexpr int kThreads = 256;        // 4 wavefronts of 64
constexpr int kPitch = kChunk + 4;   // LDS row pitch (floats): 16 lanes x b128 cover all 64 banks once
constexpr int kInvalidTap = -(1 << 29);

__device__ __forceinline__ int uniform(int v) { return __builtin_amdgcn_readfirstlane(v); }

// ---------------------------------------------------------------------------
// Preparation: tap table and filter re-layout (tiny, one launch per call)
// ---------------------------------------------------------------------------
//
// Tap table: entry g of the reduction index (channel-like index a, filter row
// r, filter column s) holds {offset, dr, ds, 0}: the BYTE offset (fp32 elements) added to a
// column's base address and the row / column displacement whose bounds decide
// whether the tap reads data or padding.
//   sign = +1 (forward, backward-filter): a = input channel c; reads
//            x[c][hb + r][wb + s]
//   sign = -1 (backward-data): a = filter k; reads dy[k][hb - r][wb - s]
// With row_pitch = col_pitch = 0 the offset names the plane only (strided
// backward-data computes the in-plane position itself).
// Entries past `len` are marked so that their bounds test always fails.
__global__ void build_tap_table(int4 *__restrict__ tab, int tab_len, int len, int RS, int S,
                                int plane, int row_pitch, int col_pitch, int sign)
{
    int g = blockIdx.x * blockDim.x + threadIdx.x;
    if (g >= tab_len) return;
    int4 e;
    if (g < len) {
        int a = g / RS, rs = g - a * RS;
        int r = rs / S, s = rs - r * S;
        e.x = 4 * (a * plane + sign * (r * row_pitch + s * col_pitch));
        e.y = sign * r;
        e.z = sign * s;
        e.w = 0;
    } else {
        e.x = 0; e.y = kInvalidTap; e.z = kInvalidTap; e.w = 0;
    }
    tab[g] = e;
}

// Filters re-laid-out as wt[chunk][Mpad][16] (zero padded): the 16-deep slice a
// work-group stages per step is one contiguous block.
//   transposed = 0: row m = filter k,  reduction index g = (c, r, s)
//   transposed = 1: row m = channel c, reduction index g = (k, r, s)
__global__ void relayout_filters(const float *__restrict__ w, float *__restrict__ wt,
                                 int M, int Mpad, int Kg, int Kgpad, int C, int RS, int transposed)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int64_t total = (int64_t)Mpad * Kgpad;
    if (i >= total) return;
    int e = (int)(i % kChunk);
    int64_t t = i / kChunk;
    int m = (int)(t % Mpad);
    int chunk = (int)(t / Mpad);
    int g = chunk * kChunk + e;
    float v = 0.f;
    if (m < M && g < Kg) {
        if (!transposed) {
            v = w[(int64_t)m * Kg + g];
        } else {
            int k = g / RS, rs = g - k * RS;
            v = w[((int64_t)k * C + m) * RS + rs];
        }
    }
    wt[i] = v;
}

// fp32 -> bf16, round to nearest even (NaN stays NaN)
// fp32 -> bfloat16 bits, round to nearest even; NaN stays a (quiet) NaN
__device__ __forceinline__ unsigned short bf16_round(float f)
{
    const unsigned u = __float_as_uint(f);
    unsigned r = (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) r = (u >> 16) | 0x40u;
    return (unsigned short)r;
}

// element access of the glue kernels: fp32 tensors, or bfloat16 tensors read exactly and written rounded
__device__ __forceinline__ float ld_elem(const float *p, int64_t i) { return p[i]; }
__device__ __forceinline__ float ld_elem(const unsigned short *p, int64_t i)
{
    return __uint_as_float((unsigned)p[i] << 16);
}
__device__ __forceinline__ float widen_elem(float v) { return v; }
__device__ __forceinline__ float widen_elem(unsigned short v) { return __uint_as_float((unsigned)v << 16); }
__device__ __forceinline__ void st_elem(float *p, int64_t i, float v) { p[i] = v; }
__device__ __forceinline__ void st_elem(unsigned short *p, int64_t i, float v) { p[i] = bf16_round(v); }

// What a forward / backward-data kernel may apply to each sum before it is stored (in this order):
//   bias: v += bias[row]        (row = output channel)
//   relu: v  = max(v, 0)
//   mask: v  = mask[n][row][pos] > 0 ? v : 0    (mask laid out like the output, samples mask_bs elements apart)
struct Epilogue {
    const float *bias;
    const void *mask;
    int64_t mask_bs;
    int relu;
    int mask_bf16;      // element type of mask: 0 = fp32, 1 = bfloat16
};

__device__ __forceinline__ float epi_apply(const Epilogue &e, float v, int row, int64_t mask_idx)
{
    if (e.bias) v += e.bias[row];
    if (e.relu) v = v > 0.f ? v : 0.f;
    if (e.mask) {
        const float m = e.mask_bf16 ? ld_elem(static_cast<const unsigned short *>(e.mask), mask_idx)
                                    : ld_elem(static_cast<const float *>(e.mask), mask_idx);
        v = m > 0.f ? v : 0.f;
    }
    return v;
}

// The epilogue on the accumulators of one 32-column block (index jn) of a wave's tile of 32 x 32 matrix blocks:
// value v of block i belongs to row row_base + 32*i + 8*(v/4) + v%4 (the accumulator layout of
// v_mfma_f32_32x32x2_f32 and v_mfma_f32_32x32x16_bf16).  The 16 loads of a block are issued before the first use,
// so their latencies overlap; rows past M (padding of the last row tile) read row M-1 and are never stored.
template <int TM, int TN>
__device__ __forceinline__ void epi_tile(const Epilogue &e, f32x16 (&acc)[TM][TN], int jn, int row_base, int M,
                                         int plane, int64_t mask_base)
{
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        int row[16];
#pragma unroll
        for (int v = 0; v < 16; ++v) row[v] = min(row_base + i * 32 + (v >> 2) * 8 + (v & 3), M - 1);
        if (e.bias) {
            float bv[16];
#pragma unroll
            for (int v = 0; v < 16; ++v) bv[v] = e.bias[row[v]];
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][jn][v] += bv[v];
        }
        if (e.relu) {
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][jn][v] = acc[i][jn][v] > 0.f ? acc[i][jn][v] : 0.f;
        }
        if (e.mask) {
            float mv[16];
            if (e.mask_bf16) {
                const unsigned short *m = static_cast<const unsigned short *>(e.mask) + mask_base;
#pragma unroll
                for (int v = 0; v < 16; ++v) mv[v] = ld_elem(m, (int64_t)row[v] * plane);
            } else {
                const float *m = static_cast<const float *>(e.mask) + mask_base;
#pragma unroll
                for (int v = 0; v < 16; ++v) mv[v] = m[(int64_t)row[v] * plane];
            }
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][jn][v] = mv[v] > 0.f ? acc[i][jn][v] : 0.f;
        }
    }
}

// The same epilogue as a pass of its own over out[n][row][pos] (samples out_bs elements apart), for the kernels
// that do not apply it themselves.
template <typename T>
__global__ void epilogue_inplace(T *__restrict__ out, int64_t out_bs, Epilogue e, int64_t total, int per_sample,
                                 FastDiv div_sample, FastDiv div_plane)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= total) return;
    const int n = (int)fastdiv((uint32_t)i, div_sample);
    const int r = (int)(i - (int64_t)n * per_sample);
    const int row = (int)fastdiv((uint32_t)r, div_plane);
    const int64_t o = (int64_t)n * out_bs + r;
    st_elem(out, o, epi_apply(e, ld_elem(out, o), row, (int64_t)n * e.mask_bs + r));
}

__global__ void narrow_to_bf16(const float *__restrict__ src, unsigned short *__restrict__ dst, int64_t n)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    dst[i] = bf16_round(src[i]);
}

// src: dense [batch][sample] fp32; dst: bf16 samples `dst_bs` elements apart (round to nearest even)
__global__ void narrow_to_bf16_strided(const float *__restrict__ src, unsigned short *__restrict__ dst, int64_t n,
                                       int64_t sample, int64_t dst_bs)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const int64_t b = i / sample;
    dst[b * dst_bs + (i - b * sample)] = bf16_round(src[i]);
}

// dst: dense [batch][sample]; src: samples `src_bs` elements apart
__global__ void widen_bf16(const unsigned short *__restrict__ src, float *__restrict__ dst, int64_t n,
                           int64_t sample, int64_t src_bs)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const int64_t b = i / sample;
    dst[i] = __uint_as_float((unsigned)src[b * src_bs + (i - b * sample)] << 16);
}

// ---------------------------------------------------------------------------
// Shared inner product: one 16-deep step of the work-group tile from LDS
// ---------------------------------------------------------------------------
//
// LDS tiles are [row][16] with pitch kPitch.  v_mfma_f32_32x32x2_f32 takes, per
// lane, A[row = lane%32][k = lane/32] and B[k = lane/32][col = lane%32].  The 16
// reduction elements of a step are fed in the order (t, 8+t), t = 0..7, so the
// lower half-wave reads elements 0..7 and the upper half 8..15 of its row: two
// b128 reads per 32-row tile.  Any order works as long as A and B agree.
template <int TM, int TN>
__device__ __forceinline__ void mma_step(const float *__restrict__ As, const float *__restrict__ Bs,
                                         int a_row0, int b_row0, int lane, f32x16 (&acc)[TM][TN])
{
    const int l32 = lane & 31, half = lane >> 5;
    f32x4 a[TM][2], b[TN][2];
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const f32x4 *p = reinterpret_cast<const f32x4 *>(As + (a_row0 + i * 32 + l32) * kPitch + half * 8);
        a[i][0] = p[0];
        a[i][1] = p[1];
    }
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const f32x4 *p = reinterpret_cast<const f32x4 *>(Bs + (b_row0 + j * 32 + l32) * kPitch + half * 8);
        b[j][0] = p[0];
        b[j][1] = p[1];
    }
#pragma unroll
    for (int t = 0; t < 8; ++t)
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i][t >> 2][t & 3], b[j][t >> 2][t & 3],
                                                                 acc[i][j], 0, 0, 0);
}

// ---------------------------------------------------------------------------
// Forward and backward-data: out[n][m][oh][ow] = sum_g A[m][g] * gather(g; n, oh, ow)
// ---------------------------------------------------------------------------
struct ColGemmArgs {
    const float *At;      // re-laid-out filters [chunks][Mpad][16]
    const int4 *tab;      // tap table
    const float *src;     // gathered tensor (x or dy)
    float *dst;           // y or dx
    int M, Mpad, nchunks;
    int OH, OW;           // extent the GEMM columns enumerate (with n): P,Q or H,W
    int LH, LW;           // extent of the gathered tensor's planes
    int ncols;            // N*OH*OW
    int src_bs, dst_bs;   // batch strides in elements
    int mul, add;         // window origin: hb = oh*mul + add, wb = ow*mul + add
    int mtiles, ntiles, tiles_per_xcd;
    FastDiv div_plane, div_ow, div_stride;
};

enum { kGatherDirect = 0, kGatherStridedBwd = 1 };

#ifdef CONVNET_PHASE_PROBE
__device__ long long *g_probe = nullptr;
#endif

template <int TM, int TN, int WM, int WN, int GATHER>
__global__ __launch_bounds__(kThreads) void colgemm_kernel(const ColGemmArgs p)
{
    constexpr int BM = TM * WM * 32, BN = TN * WN * 32;
    constexpr int EPT = BN / 16;             // gathered elements per thread per step
    constexpr int A4 = BM * 4;               // float4 loads of the filter slice per step
    constexpr int A4T = (A4 + kThreads - 1) / kThreads;
    static_assert(WM * WN == 4, "four waves per work-group");
    static_assert(BN >= 64 && (kThreads % BN == 0 || BN % kThreads == 0), "column roles");

    __shared__ __attribute__((aligned(16))) float As[2][BM * kPitch];
    __shared__ __attribute__((aligned(16))) float Bs[2][BN * kPitch];

    // Work-groups are dealt round-robin to the 8 XCDs.  Each XCD takes one
    // contiguous eighth of the tile list (row tiles fastest), so the row tiles
    // of a column tile share its gathered slice through one L2 and no XCD
    // holds more than ceil(tiles / 8) tiles.
    const int bid = blockIdx.x;
    const int idx = bid >> 3;
    const int tile = (bid & 7) * p.tiles_per_xcd + idx;
    if (idx >= p.tiles_per_xcd || tile >= p.mtiles * p.ntiles) return;
    const int mt = tile % p.mtiles, nt = tile / p.mtiles;
    const int m0 = mt * BM, n0 = nt * BN;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = uniform(tid >> 6);
    const int wm = wave / WN, wn = wave % WN;

    // --- gather role: one fixed GEMM column per thread, EPT taps of each step
    const int jc = tid % BN;
    const int grp = uniform(tid / BN);       // which EPT-wide part of the 16 taps
    const int j = n0 + jc;
    int hb, wb, base;
    {
        const bool colok = j < p.ncols;
        const int jj = colok ? j : 0;
        const int n = (int)fastdiv((uint32_t)jj, p.div_plane);
        const int rem = jj - n * (p.OH * p.OW);
        const int oh = (int)fastdiv((uint32_t)rem, p.div_ow);
        const int ow = rem - oh * p.OW;
        hb = oh * p.mul + p.add;
        wb = ow * p.mul + p.add;
        if (GATHER == kGatherDirect) base = 4 * (n * p.src_bs + hb * p.LW + wb);   // bytes
        else base = 4 * (n * p.src_bs);
        if (!colok) { hb = kInvalidTap; wb = kInvalidTap; }
    }

    f32x4 areg[A4T];
    float breg[EPT];
    bool bok[EPT];
    int4 tap[EPT];            // table entries of the step that is loaded next (wave-uniform, scalar registers)
    const char *src_bytes = reinterpret_cast<const char *>(p.src);

    // The table is padded by two steps, so fetching one step past the end is harmless.
    auto fetch_taps = [&](int chunk) {
        const int4 *t = p.tab + chunk * kChunk + grp * EPT;
#pragma unroll
        for (int e = 0; e < EPT; ++e) tap[e] = t[e];
    };
    auto slot_a = [&](int chunk) {
        const f32x4 *ablk = reinterpret_cast<const f32x4 *>(p.At + ((size_t)chunk * p.Mpad + m0) * kChunk);
#pragma unroll
        for (int i = 0; i < A4T; ++i) {
            int idx = tid + i * kThreads;
            if (A4 % kThreads == 0 || idx < A4) areg[i] = ablk[idx];
        }
    };
    auto slot_b = [&](int e) {
        bool ok;
        int off;
        if (GATHER == kGatherDirect) {
            const int hh = hb + tap[e].y, ww = wb + tap[e].z;
            ok = ((unsigned)hh < (unsigned)p.LH) & ((unsigned)ww < (unsigned)p.LW);
            off = base + tap[e].x;
        } else {
            // backward-data with stride > 1: output row h receives tap r only
            // from the window row (h + pad - r)/stride, when that divides
            const int th = hb + tap[e].y, tw = wb + tap[e].z;
            ok = (th >= 0) & (tw >= 0);
            const int ph = (int)fastdiv((uint32_t)(ok ? th : 0), p.div_stride);
            const int qw = (int)fastdiv((uint32_t)(ok ? tw : 0), p.div_stride);
            ok = ok & (ph * (int)p.div_stride.d == th) & (qw * (int)p.div_stride.d == tw) &
                 (ph < p.LH) & (qw < p.LW);
            off = base + tap[e].x + 4 * (ph * p.LW + qw);
        }
        // the load is always issued (address 0 when the tap is padding); the
        // zero is substituted when the value is staged, after the MFMAs
        breg[e] = *reinterpret_cast<const float *>(src_bytes + (uint32_t)(ok ? off : 0));
        bok[e] = ok;
    };

    auto store_step = [&](int buf) {
#pragma unroll
        for (int i = 0; i < A4T; ++i) {
            int idx = tid + i * kThreads;
            if (A4 % kThreads == 0 || idx < A4)
                *reinterpret_cast<f32x4 *>(&As[buf][(idx >> 2) * kPitch + (idx & 3) * 4]) = areg[i];
        }
        float *brow = &Bs[buf][jc * kPitch + grp * EPT];
#pragma unroll
        for (int e = 0; e < EPT; e += 4) {
            f32x4 v = {bok[e] ? breg[e] : 0.f, bok[e + 1] ? breg[e + 1] : 0.f, bok[e + 2] ? breg[e + 2] : 0.f,
                       bok[e + 3] ? breg[e + 3] : 0.f};
            *reinterpret_cast<f32x4 *>(brow + e) = v;
        }
    };

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int jn = 0; jn < TN; ++jn)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][jn][v] = 0.f;

    const int l32_ = lane & 31, half_ = lane >> 5;
    const int a_frag = (wm * TM * 32 + l32_) * kPitch + half_ * 8;
    const int b_frag = (wn * TN * 32 + l32_) * kPitch + half_ * 8;
    constexpr int NMMA = 8 * TM * TN;
    constexpr int NSLOT = EPT + 2;                              // filter slice, EPT taps, table prefetch
    constexpr int SPM = (NSLOT + NMMA - 5) / (NMMA - 4);

    fetch_taps(0);
    slot_a(0);
#pragma unroll
    for (int e = 0; e < EPT; ++e) slot_b(e);
    store_step(0);
    fetch_taps(1);
    __syncthreads();
    for (int chunk = 0; chunk < p.nchunks - 1; ++chunk) {
        const int buf = chunk & 1;
        f32x4 fa[TM][2], fb[TN][2];
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const f32x4 *q = reinterpret_cast<const f32x4 *>(&As[buf][a_frag + i * 32 * kPitch]);
            fa[i][0] = q[0]; fa[i][1] = q[1];
        }
#pragma unroll
        for (int jn = 0; jn < TN; ++jn) {
            const f32x4 *q = reinterpret_cast<const f32x4 *>(&Bs[buf][b_frag + jn * 32 * kPitch]);
            fb[jn][0] = q[0]; fb[jn][1] = q[1];
        }
        __builtin_amdgcn_sched_barrier(0);
        // the next step's loads issue in the shadow of this step's matrix instructions
#pragma unroll
        for (int m = 0; m < NMMA; ++m) {
            const int t = m / (TM * TN), i = (m / TN) % TM, jn = m % TN;
            acc[i][jn] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[i][t >> 2][t & 3], fb[jn][t >> 2][t & 3],
                                                              acc[i][jn], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int q = m * SPM; q < (m + 1) * SPM && q < NSLOT; ++q) {
                if (q == 0) slot_a(chunk + 1);
                else if (q - 1 < EPT) slot_b(q - 1);
                else fetch_taps(chunk + 2);
            }
            if (m * SPM < NSLOT) __builtin_amdgcn_sched_barrier(0);
        }
        store_step(buf ^ 1);
        __syncthreads();
    }
    mma_step<TM, TN>(As[(p.nchunks - 1) & 1], Bs[(p.nchunks - 1) & 1], wm * TM * 32, wn * TN * 32, lane, acc);

    // --- epilogue.  Accumulator register v of lane l holds row
    // 8*(v/4) + 4*(l/32) + v%4 and column l%32 of its 32 x 32 tile.
    const int l32 = lane & 31, half = lane >> 5;
    const int plane = p.OH * p.OW;
#pragma unroll
    for (int jn = 0; jn < TN; ++jn) {
        const int col = n0 + (wn * TN + jn) * 32 + l32;
        if (col >= p.ncols) continue;
        const int n = (int)fastdiv((uint32_t)col, p.div_plane);
        const int rem = col - n * plane;
        float *out = p.dst + (size_t)n * p.dst_bs + rem;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int row0 = m0 + (wm * TM + i) * 32 + half * 4;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = row0 + (v >> 2) * 8 + (v & 3);
                if (row < p.M) out[(size_t)row * plane] = acc[i][jn][v];
            }
        }
    }
}

// ---------------------------------------------------------------------------
// Forward / stride-1 backward-data when the reduction channel count is a
// multiple of 16: each 16-deep step is one filter tap (r, s) and 16 consecutive
// channels, so the padding test and the address of a thread's column are
// computed once per step and its taps differ only by the channel stride.
// Steps run channel-block-major, taps inside ((cb, r, s) order) so the nine or
// twenty-five shifted reads of a channel block hit the same cache lines.
// ---------------------------------------------------------------------------
struct ColGemmFastArgs {
    const float *At;      // filters as [cb][r][s][Mpad][KC channels]
    const float *src;
    float *dst;
    int M, Mpad;
    int cblocks, R, S;    // reduction: cblocks * R * S steps of KC channels
    int sign;             // +1 forward (reads hb + r), -1 backward-data (reads hb - r)
    int plane_bytes;      // LH*LW*4: channel stride of the gathered tensor
    int OH, OW, LH, LW;
    int ncols, src_bs, dst_bs, mul, add;
    int mtiles, ntiles, tiles_per_xcd;
    int ksplit, steps_per_split;   // the reduction steps are cut into ksplit ranges (1 = whole)
    float *part;                   // ksplit > 1: partial outputs [ksplit][N][M][OH*OW], summed by reduce_split_outputs
    int out_bf16;                  // bf16 kernel only: dst holds bfloat16 (each sum rounded to nearest even)
    // columns of a grouped layer in one launch (fp32 kernels): column g reads src + g * src_gs, the filter copy
    // At + g * at_gs, writes dst + g * dst_gs and the partials part + g * part_gs (all in floats)
    int groups;
    int64_t src_gs, dst_gs, at_gs, part_gs;
    // applied where the final sums are stored (this kernel when ksplit == 1 and epi_on, else the split-sum kernel)
    int epi_on;
    Epilogue epi;
    FastDiv div_plane, div_ow, div_rs, div_s;
};

// KC = reduction depth of one step (16 or 32 channels of one tap).  LDS is
// dynamic: 2 * (BM + BN) * (KC + 4) floats.
template <int TM, int TN, int WM, int WN, int KC>
__global__ __launch_bounds__(kThreads, 2) void colgemm_fast_kernel(const ColGemmFastArgs p)
{
    constexpr int BM = TM * WM * 32, BN = TN * WN * 32;
    constexpr int PITCH = KC + 4;            // 16 lanes x b128 still cover all banks once (20 and 36 both do)
    constexpr int HALFK = KC / 2;            // reduction elements each half-wave feeds
    constexpr int NF = HALFK / 4;            // b128 reads per 32-row fragment
    constexpr int EPT = BN * KC / kThreads;  // gathered channels per thread per step
    constexpr int A4 = BM * KC / 4;
    constexpr int A4T = (A4 + kThreads - 1) / kThreads;
    static_assert(WM * WN == 4, "four waves per work-group");
    static_assert(KC == 16 || KC == 32, "step depth");

    extern __shared__ __attribute__((aligned(16))) float lds_fast[];
    float *const As0 = lds_fast;
    float *const Bs0 = lds_fast + 2 * BM * PITCH;

    const int bid = blockIdx.x;
    const int idx = bid >> 3;
    const int unit = (bid & 7) * p.tiles_per_xcd + idx;
    const int ntile = p.mtiles * p.ntiles;
    if (idx >= p.tiles_per_xcd || unit >= ntile * p.ksplit * p.groups) return;
    const int grp_col = unit / (ntile * p.ksplit);              // column of a grouped layer
    const int unit_c = unit - grp_col * (ntile * p.ksplit);
    const int ks = unit_c / ntile;
    const int tile = unit_c - ks * ntile;
    const float *const At_c = p.At + (size_t)grp_col * p.at_gs;
    const float *const src_c = p.src + (size_t)grp_col * p.src_gs;
    float *const dst_c = p.dst + (size_t)grp_col * p.dst_gs;
    float *const part_c = p.part + (size_t)grp_col * p.part_gs;
    const int mt = tile % p.mtiles, nt = tile / p.mtiles;
    const int m0 = mt * BM, n0 = nt * BN;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = uniform(tid >> 6);
    const int wm = wave / WN, wn = wave % WN;

    const int jc = tid % BN;
    const int grp = uniform(tid / BN);
    int hb, wb, base;
    {
        const int j = n0 + jc;
        const bool colok = j < p.ncols;
        const int jj = colok ? j : 0;
        const int n = (int)fastdiv((uint32_t)jj, p.div_plane);
        const int rem = jj - n * (p.OH * p.OW);
        const int oh = (int)fastdiv((uint32_t)rem, p.div_ow);
        const int ow = rem - oh * p.OW;
        hb = oh * p.mul + p.add;
        wb = ow * p.mul + p.add;
        base = 4 * (n * p.src_bs + hb * p.LW + wb) + grp * EPT * p.plane_bytes;
        if (!colok) { hb = kInvalidTap; wb = kInvalidTap; }
    }
    const char *src_bytes = reinterpret_cast<const char *>(src_c);
    const size_t a_step = (size_t)p.Mpad * (KC / 4);          // f32x4 per step
    const int step_begin = ks * p.steps_per_split;
    const int nsteps = min(p.cblocks * p.R * p.S - step_begin, p.steps_per_split);
    const f32x4 *a_ptr = reinterpret_cast<const f32x4 *>(At_c + (size_t)m0 * KC) + tid + step_begin * a_step;

    // Data of step t lives in register set t & 1 and LDS buffer t & 1.  While step s is multiplied out of
    // buffer s & 1, the loads of step s + 2 are issued into set s & 1 (free since its contents went to LDS
    // during step s - 1) and the values of step s + 1, loaded a whole step earlier, are written from the other
    // set into the other buffer -- all of it in slots between the matrix instructions, so that between two
    // steps only the barrier and the first fragment reads remain.
    f32x4 areg[2][A4T];
    float breg[2][EPT];
    bool bok[2];
    int a0 = 0;
    // next step to load: tap (r, s), channel-block byte offset
    int r, s, cboff;
    {
        const int cb = (int)fastdiv((uint32_t)step_begin, p.div_rs);
        const int rs = step_begin - cb * (p.R * p.S);
        r = (int)fastdiv((uint32_t)rs, p.div_s);
        s = rs - r * p.S;
        cboff = cb * KC * p.plane_bytes;
    }

    auto slot_tap = [&](int set) {   // padding test and column address of tap (r, s)
        const int dr = p.sign * r, ds = p.sign * s;
        const int hh = hb + dr, ww = wb + ds;
        bok[set] = ((unsigned)hh < (unsigned)p.LH) & ((unsigned)ww < (unsigned)p.LW);
        a0 = bok[set] ? base + cboff + 4 * (dr * p.LW + ds) : 0;
        s += 1;
        const bool ws = s == p.S;
        s = ws ? 0 : s;
        r += ws ? 1 : 0;
        const bool wr = r == p.R;
        r = wr ? 0 : r;
        cboff += wr ? KC * p.plane_bytes : 0;
    };
    auto slot_a = [&](int set, int i) {       // filter slice: contiguous block
        if (A4 % kThreads == 0 || tid + i * kThreads < A4) areg[set][i] = a_ptr[i * kThreads];
        if (i == A4T - 1) a_ptr += a_step;
    };
    auto slot_b = [&](int set, int e) {       // one channel of the gathered column
        breg[set][e] = *reinterpret_cast<const float *>(src_bytes + (uint32_t)(a0 + e * p.plane_bytes));
    };
    auto load_step = [&](int set) {
        slot_tap(set);
#pragma unroll
        for (int i = 0; i < A4T; ++i) slot_a(set, i);
#pragma unroll
        for (int e = 0; e < EPT; ++e) slot_b(set, e);
    };
    auto store_a = [&](int set, int i) {      // one 16-byte piece of the filter slice into LDS buffer `set`
        float *As = As0 + set * BM * PITCH;
        const int q = tid + i * kThreads;
        if (A4 % kThreads == 0 || q < A4)
            *reinterpret_cast<f32x4 *>(&As[(q / (KC / 4)) * PITCH + (q % (KC / 4)) * 4]) = areg[set][i];
    };
    auto store_b = [&](int set, int g) {      // four gathered channels into LDS buffer `set`, zeros for a padding tap
        float *brow = Bs0 + set * BN * PITCH + jc * PITCH + grp * EPT;
        const int e = 4 * g;
        f32x4 v = {bok[set] ? breg[set][e] : 0.f, bok[set] ? breg[set][e + 1] : 0.f,
                   bok[set] ? breg[set][e + 2] : 0.f, bok[set] ? breg[set][e + 3] : 0.f};
        *reinterpret_cast<f32x4 *>(brow + e) = v;
    };
    auto store_step = [&](int set) {
#pragma unroll
        for (int i = 0; i < A4T; ++i) store_a(set, i);
#pragma unroll
        for (int g = 0; g < EPT / 4; ++g) store_b(set, g);
    };

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int jn = 0; jn < TN; ++jn)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][jn][v] = 0.f;

    const int l32 = lane & 31, half = lane >> 5;
    const int a_frag = (wm * TM * 32 + l32) * PITCH + half * HALFK;
    const int b_frag = (wn * TN * 32 + l32) * PITCH + half * HALFK;
    constexpr int NMMA = HALFK * TM * TN;
    constexpr int NLOAD = 1 + A4T + EPT;                        // load slots: tap, filter slice, EPT channels
    constexpr int NSTORE = A4T + EPT / 4;                       // store slots
    constexpr int SPM = (NLOAD + NSTORE + NMMA - 3) / (NMMA - 2);   // slots after each matrix instruction

#ifdef CONVNET_PHASE_PROBE
    const long long pr_t0 = __builtin_readcyclecounter();
    const long long pr_rt0 = wall_clock64();
#endif
    load_step(0);
    store_step(0);
    if (nsteps > 1) load_step(1);
    __syncthreads();
#ifdef CONVNET_PHASE_PROBE
    const long long pr_rt1 = wall_clock64();
#endif
    // One step out of LDS buffer `par`.  par and mode are compile-time constants: the register sets stay in
    // registers and the slot stream has no branches, so the waits before the LDS writes count only the loads
    // issued a step earlier.  mode 2: loads of step + 2 and stores of step + 1; 1: stores only; 0: neither.
    auto do_step = [&](auto par_c, auto mode_c) {
        constexpr int par = decltype(par_c)::value, mode = decltype(mode_c)::value;
        const float *As = As0 + par * BM * PITCH, *Bs = Bs0 + par * BN * PITCH;
        f32x4 fa[TM][NF], fb[TN][NF];
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const f32x4 *q = reinterpret_cast<const f32x4 *>(&As[a_frag + i * 32 * PITCH]);
#pragma unroll
            for (int f = 0; f < NF; ++f) fa[i][f] = q[f];
        }
#pragma unroll
        for (int jn = 0; jn < TN; ++jn) {
            const f32x4 *q = reinterpret_cast<const f32x4 *>(&Bs[b_frag + jn * 32 * PITCH]);
#pragma unroll
            for (int f = 0; f < NF; ++f) fb[jn][f] = q[f];
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int m = 0; m < NMMA; ++m) {
            const int t = m / (TM * TN), i = (m / TN) % TM, jn = m % TN;
            acc[i][jn] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[i][t >> 2][t & 3], fb[jn][t >> 2][t & 3],
                                                              acc[i][jn], 0, 0, 0);
            if (mode > 0 && m * SPM < NLOAD + NSTORE) {
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int q = m * SPM; q < (m + 1) * SPM && q < NLOAD + NSTORE; ++q) {
                    if (q < NLOAD) {
                        if (mode == 2) {
                            if (q == 0) slot_tap(par);
                            else if (q - 1 < A4T) slot_a(par, q - 1);
                            else slot_b(par, q - 1 - A4T);
                        }
                    } else {
                        const int w = q - NLOAD;
                        if (w < A4T) store_a(par ^ 1, w);
                        else store_b(par ^ 1, w - A4T);
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        if (mode > 0) __syncthreads();
    };
    using P0 = std::integral_constant<int, 0>;
    using P1 = std::integral_constant<int, 1>;
    using M2 = std::integral_constant<int, 2>;
    int step = 0;
    for (; step + 3 < nsteps; step += 2) {
        do_step(P0{}, M2{});
        do_step(P1{}, M2{});
    }
    const int rest = nsteps - step;                 // 1, 2 or 3 steps left, the first in buffer 0
    if (rest == 3) {
        do_step(P0{}, M2{});
        do_step(P1{}, P1{});
        do_step(P0{}, P0{});
    } else if (rest == 2) {
        do_step(P0{}, P1{});
        do_step(P1{}, P0{});
    } else if (rest == 1) {
        do_step(P0{}, P0{});
    }
#ifdef CONVNET_PHASE_PROBE
    if (tid == 0 && g_probe) {
        long long *o = g_probe + (size_t)bid * 8;
        o[0] = pr_t0; o[1] = __builtin_readcyclecounter(); o[2] = pr_rt0; o[3] = wall_clock64(); o[5] = pr_rt1;
        o[6] = __builtin_amdgcn_s_getreg(4 | (0 << 6) | (31 << 11));
        o[7] = __builtin_amdgcn_s_getreg(20 | (0 << 6) | (31 << 11));
    }
#endif

    const int plane = p.OH * p.OW;
#pragma unroll
    for (int jn = 0; jn < TN; ++jn) {
        const int col = n0 + (wn * TN + jn) * 32 + l32;
        if (col >= p.ncols) continue;
        const int n = (int)fastdiv((uint32_t)col, p.div_plane);
        const int rem = col - n * plane;
        float *out = p.ksplit > 1 ? part_c + ((size_t)ks * (p.ncols / plane) + n) * ((size_t)p.M * plane) + rem
                                  : dst_c + (size_t)n * p.dst_bs + rem;
        if (p.epi_on && p.ksplit == 1)            // one column only; split sums get it in reduce_split_outputs
            epi_tile<TM, TN>(p.epi, acc, jn, m0 + wm * TM * 32 + half * 4, p.M, plane,
                             (int64_t)n * p.epi.mask_bs + rem);
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int row0 = m0 + (wm * TM + i) * 32 + half * 4;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = row0 + (v >> 2) * 8 + (v & 3);
                if (row < p.M) out[(size_t)row * plane] = acc[i][jn][v];
            }
        }
    }
#ifdef CONVNET_PHASE_PROBE
    __builtin_amdgcn_s_waitcnt(0);
    if (tid == 0 && g_probe) g_probe[(size_t)bid * 8 + 4] = wall_clock64();
#endif
}

// ---------------------------------------------------------------------------
// The same walk as colgemm_fast_kernel for GEMM views of 33..48 rows (backward-
// data of a 48-channel column): 32-row matrix tiles would pad 48 rows to 64, so
// this kernel works in 16 x 16 blocks on v_mfma_f32_16x16x4_f32.  A work-group
// covers 48 rows x 256 columns, a wave 48 x 64 (3 x 4 blocks).  Per lane the
// instruction takes A[row = lane%16][k = lane/16] and B[k = lane/16][col =
// lane%16] and returns D[row = 4*(lane/16) + v][col = lane%16], v = 0..3.  A lane
// reads the four consecutive reduction elements 4*(lane/16).. of its row with one
// b128 and feeds element t to the t-th instruction, so the 16 elements of a step
// are consumed in the order (t, 4+t, 8+t, 12+t) on both operands.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(kThreads, 3) void colgemm_rows48_kernel(const ColGemmFastArgs p)
{
    constexpr int BM = 48, BN = 256, KC = 16, PITCH = KC + 4;
    constexpr int TM = 3, TN = 4;            // 16 x 16 blocks per wave
    constexpr int EPT = KC;                  // a thread gathers all 16 channels of its column
    constexpr int A4 = BM * KC / 4;          // 192 vectors of the filter slice per step

    extern __shared__ __attribute__((aligned(16))) float lds_fast[];
    float *const As0 = lds_fast;
    float *const Bs0 = lds_fast + 2 * BM * PITCH;

    const int bid = blockIdx.x;
    const int idx = bid >> 3;
    const int unit = (bid & 7) * p.tiles_per_xcd + idx;
    const int ntile = p.mtiles * p.ntiles;
    if (idx >= p.tiles_per_xcd || unit >= ntile * p.ksplit * p.groups) return;
    const int grp_col = unit / (ntile * p.ksplit);              // column of a grouped layer
    const int unit_c = unit - grp_col * (ntile * p.ksplit);
    const int ks = unit_c / ntile;
    const int tile = unit_c - ks * ntile;
    const float *const At_c = p.At + (size_t)grp_col * p.at_gs;
    const float *const src_c = p.src + (size_t)grp_col * p.src_gs;
    float *const dst_c = p.dst + (size_t)grp_col * p.dst_gs;
    float *const part_c = p.part + (size_t)grp_col * p.part_gs;
    const int mt = tile % p.mtiles, nt = tile / p.mtiles;
    const int m0 = mt * BM, n0 = nt * BN;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wn = uniform(tid >> 6);
    const int jc = tid;
    int hb, wb, base;
    {
        const int j = n0 + jc;
        const bool colok = j < p.ncols;
        const int jj = colok ? j : 0;
        const int n = (int)fastdiv((uint32_t)jj, p.div_plane);
        const int rem = jj - n * (p.OH * p.OW);
        const int oh = (int)fastdiv((uint32_t)rem, p.div_ow);
        const int ow = rem - oh * p.OW;
        hb = oh * p.mul + p.add;
        wb = ow * p.mul + p.add;
        base = 4 * (n * p.src_bs + hb * p.LW + wb);
        if (!colok) { hb = kInvalidTap; wb = kInvalidTap; }
    }
    const char *src_bytes = reinterpret_cast<const char *>(src_c);
    const size_t a_step = (size_t)p.Mpad * (KC / 4);
    const int step_begin = ks * p.steps_per_split;
    const int nsteps = min(p.cblocks * p.R * p.S - step_begin, p.steps_per_split);
    const f32x4 *a_ptr = reinterpret_cast<const f32x4 *>(At_c + (size_t)m0 * KC) + tid + step_begin * a_step;

    // register set t & 1 and LDS buffer t & 1 hold step t (two-set pipeline of colgemm_fast_kernel)
    f32x4 areg[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
    float breg[2][EPT];
    bool bok[2];
    int a0 = 0;
    int r, s, cboff;
    {
        const int cb = (int)fastdiv((uint32_t)step_begin, p.div_rs);
        const int rs = step_begin - cb * (p.R * p.S);
        r = (int)fastdiv((uint32_t)rs, p.div_s);
        s = rs - r * p.S;
        cboff = cb * KC * p.plane_bytes;
    }
    auto slot_tap = [&](int set) {
        const int dr = p.sign * r, ds = p.sign * s;
        const int hh = hb + dr, ww = wb + ds;
        bok[set] = ((unsigned)hh < (unsigned)p.LH) & ((unsigned)ww < (unsigned)p.LW);
        a0 = bok[set] ? base + cboff + 4 * (dr * p.LW + ds) : 0;
        s += 1;
        const bool ws = s == p.S;
        s = ws ? 0 : s;
        r += ws ? 1 : 0;
        const bool wr = r == p.R;
        r = wr ? 0 : r;
        cboff += wr ? KC * p.plane_bytes : 0;
    };
    auto slot_a = [&](int set) {
        if (tid < A4) areg[set] = a_ptr[0];
        a_ptr += a_step;
    };
    auto slot_b = [&](int set, int e) {
        breg[set][e] = *reinterpret_cast<const float *>(src_bytes + (uint32_t)(a0 + e * p.plane_bytes));
    };
    auto load_step = [&](int set) {
        slot_tap(set);
        slot_a(set);
#pragma unroll
        for (int e = 0; e < EPT; ++e) slot_b(set, e);
    };
    auto store_a = [&](int set) {
        float *As = As0 + set * BM * PITCH;
        if (tid < A4) *reinterpret_cast<f32x4 *>(&As[(tid >> 2) * PITCH + (tid & 3) * 4]) = areg[set];
    };
    auto store_b = [&](int set, int g) {
        float *brow = Bs0 + set * BN * PITCH + jc * PITCH;
        const int e = 4 * g;
        f32x4 v = {bok[set] ? breg[set][e] : 0.f, bok[set] ? breg[set][e + 1] : 0.f,
                   bok[set] ? breg[set][e + 2] : 0.f, bok[set] ? breg[set][e + 3] : 0.f};
        *reinterpret_cast<f32x4 *>(brow + e) = v;
    };
    auto store_step = [&](int set) {
        store_a(set);
#pragma unroll
        for (int g = 0; g < EPT / 4; ++g) store_b(set, g);
    };

    f32x4 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int jn = 0; jn < TN; ++jn) acc[i][jn] = f32x4{0.f, 0.f, 0.f, 0.f};

    const int l16 = lane & 15, kq = lane >> 4;
    const int a_frag = l16 * PITCH + kq * 4;
    const int b_frag = (wn * TN * 16 + l16) * PITCH + kq * 4;
    constexpr int NMMA = 4 * TM * TN;
    constexpr int NLOAD = 2 + EPT, NSTORE = 1 + EPT / 4;

    load_step(0);
    store_step(0);
    if (nsteps > 1) load_step(1);
    __syncthreads();
    // mode 2: loads of step + 2 and stores of step + 1; 1: stores only; 0: neither (par, mode compile-time)
    auto do_step = [&](auto par_c, auto mode_c) {
        constexpr int par = decltype(par_c)::value, mode = decltype(mode_c)::value;
        const float *As = As0 + par * BM * PITCH, *Bs = Bs0 + par * BN * PITCH;
        f32x4 fa[TM], fb[TN];
#pragma unroll
        for (int i = 0; i < TM; ++i) fa[i] = *reinterpret_cast<const f32x4 *>(&As[a_frag + i * 16 * PITCH]);
#pragma unroll
        for (int jn = 0; jn < TN; ++jn) fb[jn] = *reinterpret_cast<const f32x4 *>(&Bs[b_frag + jn * 16 * PITCH]);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int m = 0; m < NMMA; ++m) {
            const int t = m / (TM * TN), i = (m / TN) % TM, jn = m % TN;
            acc[i][jn] = __builtin_amdgcn_mfma_f32_16x16x4f32(fa[i][t], fb[jn][t], acc[i][jn], 0, 0, 0);
            if (mode > 0 && m < NLOAD + NSTORE) {
                __builtin_amdgcn_sched_barrier(0);
                if (m < NLOAD) {
                    if (mode == 2) {
                        if (m == 0) slot_tap(par);
                        else if (m == 1) slot_a(par);
                        else slot_b(par, m - 2);
                    }
                } else {
                    if (m == NLOAD) store_a(par ^ 1);
                    else store_b(par ^ 1, m - NLOAD - 1);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        if (mode > 0) __syncthreads();
    };
    using P0 = std::integral_constant<int, 0>;
    using P1 = std::integral_constant<int, 1>;
    using M2 = std::integral_constant<int, 2>;
    int step = 0;
    for (; step + 3 < nsteps; step += 2) {
        do_step(P0{}, M2{});
        do_step(P1{}, M2{});
    }
    const int rest = nsteps - step;
    if (rest == 3) {
        do_step(P0{}, M2{});
        do_step(P1{}, P1{});
        do_step(P0{}, P0{});
    } else if (rest == 2) {
        do_step(P0{}, P1{});
        do_step(P1{}, P0{});
    } else if (rest == 1) {
        do_step(P0{}, P0{});
    }

    const int plane = p.OH * p.OW;
#pragma unroll
    for (int jn = 0; jn < TN; ++jn) {
        const int col = n0 + (wn * TN + jn) * 16 + l16;
        if (col >= p.ncols) continue;
        const int n = (int)fastdiv((uint32_t)col, p.div_plane);
        const int rem = col - n * plane;
        float *out = p.ksplit > 1 ? part_c + ((size_t)ks * (p.ncols / plane) + n) * ((size_t)p.M * plane) + rem
                                  : dst_c + (size_t)n * p.dst_bs + rem;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int row = m0 + i * 16 + kq * 4 + v;
                if (row < p.M) out[(size_t)row * plane] = acc[i][jn][v];
            }
    }
}

// ---------------------------------------------------------------------------
// bf16 inputs, fp32 accumulation: the same walk as colgemm_fast_kernel (one
// filter tap x KC consecutive channels per step, one padding test and one base
// address per thread and step) on v_mfma_f32_32x32x16_bf16.  A lane feeds 8
// consecutive channels of its row per instruction, so the LDS tiles are
// [row][KC bf16] with 16 bytes of padding per row and every fragment read is one
// b128.  In NCHW a column's channels lie a plane apart, which would make every
// gathered element its own 2-byte load; block_channels_bf16 therefore first
// copies the gathered tensor into [n][channel block of 16][h][w][16 channels],
// so that 8 channels of one position are one 16-byte load that goes to LDS as it
// is.  KC (channels per step) is 16, 32, 48 or 64.
// ---------------------------------------------------------------------------
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

template <int TM, int TN, int WM, int WN, int KC>
__global__ __launch_bounds__(kThreads, 2) void colgemm_bf16_kernel(const ColGemmFastArgs p)
{
    constexpr int BM = TM * WM * 32, BN = TN * WN * 32;
    constexpr int PITCHB = KC * 2 + 16;      // bytes per LDS row
    constexpr int NK = KC / 16;              // matrix instructions per 32x32 tile and step
    constexpr int EPT = BN * KC / kThreads;  // gathered channels per thread per step
    constexpr int NV = EPT / 8;              // ... as 16-byte vectors
    constexpr int A4 = BM * KC / 8;          // 16-byte vectors of the filter slice per step
    constexpr int A4T = (A4 + kThreads - 1) / kThreads;
    static_assert(WM * WN == 4, "four waves per work-group");
    static_assert(KC % 16 == 0 && KC <= 64, "step depth");
    static_assert(EPT % 8 == 0, "a thread stages whole 16-byte groups");

    extern __shared__ __attribute__((aligned(16))) float lds_fast[];
    char *const As0 = reinterpret_cast<char *>(lds_fast);
    char *const Bs0 = As0 + 2 * BM * PITCHB;

    const int bid = blockIdx.x;
    const int idx = bid >> 3;
    const int unit = (bid & 7) * p.tiles_per_xcd + idx;
    const int ntile = p.mtiles * p.ntiles;
    if (idx >= p.tiles_per_xcd || unit >= ntile * p.ksplit) return;
    const int ks = unit / ntile;
    const int tile = unit - ks * ntile;
    const int mt = tile % p.mtiles, nt = tile / p.mtiles;
    const int m0 = mt * BM, n0 = nt * BN;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = uniform(tid >> 6);
    const int wm = wave / WN, wn = wave % WN;

    const int jc = tid % BN;
    const int grp = uniform(tid / BN);
    int hb, wb, base;                        // base: byte offset of this column at tap (0, 0) in channel block 0
    {
        const int j = n0 + jc;
        const bool colok = j < p.ncols;
        const int jj = colok ? j : 0;
        const int n = (int)fastdiv((uint32_t)jj, p.div_plane);
        const int rem = jj - n * (p.OH * p.OW);
        const int oh = (int)fastdiv((uint32_t)rem, p.div_ow);
        const int ow = rem - oh * p.OW;
        hb = oh * p.mul + p.add;
        wb = ow * p.mul + p.add;
        base = 32 * (n * p.src_bs + hb * p.LW + wb);          // src_bs: 32-byte position blocks per sample
        if (!colok) { hb = kInvalidTap; wb = kInvalidTap; }
    }
    int voff[NV];                            // this thread's vectors inside a step: channels grp*EPT + 8v ..+7
#pragma unroll
    for (int v = 0; v < NV; ++v) {
        const int c = grp * EPT + 8 * v;
        voff[v] = (c >> 4) * p.plane_bytes + (c & 15) * 2;
    }
    const char *src_bytes = reinterpret_cast<const char *>(p.src);
    const size_t a_step = (size_t)p.Mpad * (KC / 8);          // 16-byte vectors per step
    const int step_begin = ks * p.steps_per_split;
    const int nsteps = min(p.cblocks * p.R * p.S - step_begin, p.steps_per_split);
    const u32x4 *a_ptr = reinterpret_cast<const u32x4 *>(p.At) + (size_t)m0 * (KC / 8) + tid + step_begin * a_step;

    // register set t & 1 and LDS buffer t & 1 hold step t (two-set pipeline of colgemm_fast_kernel)
    u32x4 areg[2][A4T];
    u32x4 breg[2][NV];
    bool bok[2];
    int a0 = 0;
    int r, s, cboff;
    {
        const int cb = (int)fastdiv((uint32_t)step_begin, p.div_rs);
        const int rs = step_begin - cb * (p.R * p.S);
        r = (int)fastdiv((uint32_t)rs, p.div_s);
        s = rs - r * p.S;
        cboff = cb * (KC / 16) * p.plane_bytes;
    }

    auto slot_tap = [&](int set) {
        const int dr = p.sign * r, ds = p.sign * s;
        const int hh = hb + dr, ww = wb + ds;
        bok[set] = ((unsigned)hh < (unsigned)p.LH) & ((unsigned)ww < (unsigned)p.LW);
        a0 = bok[set] ? base + cboff + 32 * (dr * p.LW + ds) : 0;
        s += 1;
        const bool ws = s == p.S;
        s = ws ? 0 : s;
        r += ws ? 1 : 0;
        const bool wr = r == p.R;
        r = wr ? 0 : r;
        cboff += wr ? (KC / 16) * p.plane_bytes : 0;
    };
    auto slot_a = [&](int set, int i) {
        if (A4 % kThreads == 0 || tid + i * kThreads < A4) areg[set][i] = a_ptr[i * kThreads];
        if (i == A4T - 1) a_ptr += a_step;
    };
    auto slot_b = [&](int set, int v) {
        breg[set][v] = *reinterpret_cast<const u32x4 *>(src_bytes + (uint32_t)(a0 + voff[v]));
    };
    auto load_step = [&](int set) {
        slot_tap(set);
#pragma unroll
        for (int i = 0; i < A4T; ++i) slot_a(set, i);
#pragma unroll
        for (int v = 0; v < NV; ++v) slot_b(set, v);
    };
    auto store_a = [&](int set, int i) {
        char *As = As0 + set * BM * PITCHB;
        const int q = tid + i * kThreads;
        if (A4 % kThreads == 0 || q < A4)
            *reinterpret_cast<u32x4 *>(As + (q / (KC / 8)) * PITCHB + (q % (KC / 8)) * 16) = areg[set][i];
    };
    auto store_b = [&](int set, int v) {
        char *brow = Bs0 + set * BN * PITCHB + jc * PITCHB + grp * EPT * 2;
        u32x4 q;
#pragma unroll
        for (int k = 0; k < 4; ++k) q[k] = bok[set] ? breg[set][v][k] : 0u;
        *reinterpret_cast<u32x4 *>(brow + v * 16) = q;
    };
    auto store_step = [&](int set) {
#pragma unroll
        for (int i = 0; i < A4T; ++i) store_a(set, i);
#pragma unroll
        for (int v = 0; v < NV; ++v) store_b(set, v);
    };

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int jn = 0; jn < TN; ++jn)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][jn][v] = 0.f;

    const int l32 = lane & 31, half = lane >> 5;
    const int a_frag = (wm * TM * 32 + l32) * PITCHB + half * 16;
    const int b_frag = (wn * TN * 32 + l32) * PITCHB + half * 16;
    constexpr int NMMA = NK * TM * TN;
    constexpr int NLOAD = 1 + A4T + NV, NSTORE = A4T + NV;
    constexpr int SPM = (NLOAD + NSTORE + (NMMA > 2 ? NMMA - 2 : 1) - 1) / (NMMA > 2 ? NMMA - 2 : 1);

    load_step(0);
    store_step(0);
    if (nsteps > 1) load_step(1);
    __syncthreads();
    // mode 2: loads of step + 2 and stores of step + 1; 1: stores only; 0: neither (par, mode compile-time)
    auto do_step = [&](auto par_c, auto mode_c) {
        constexpr int par = decltype(par_c)::value, mode = decltype(mode_c)::value;
        const char *As = As0 + par * BM * PITCHB, *Bs = Bs0 + par * BN * PITCHB;
        u32x4 fa[TM][NK], fb[TN][NK];
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int t = 0; t < NK; ++t)
                fa[i][t] = *reinterpret_cast<const u32x4 *>(As + a_frag + i * 32 * PITCHB + t * 32);
#pragma unroll
        for (int jn = 0; jn < TN; ++jn)
#pragma unroll
            for (int t = 0; t < NK; ++t)
                fb[jn][t] = *reinterpret_cast<const u32x4 *>(Bs + b_frag + jn * 32 * PITCHB + t * 32);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int m = 0; m < NMMA; ++m) {
            const int t = m / (TM * TN), i = (m / TN) % TM, jn = m % TN;
            acc[i][jn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fa[i][t]),
                                                                 __builtin_bit_cast(bf16x8, fb[jn][t]),
                                                                 acc[i][jn], 0, 0, 0);
            if (mode > 0 && m * SPM < NLOAD + NSTORE) {
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int q = m * SPM; q < (m + 1) * SPM && q < NLOAD + NSTORE; ++q) {
                    if (q < NLOAD) {
                        if (mode == 2) {
                            if (q == 0) slot_tap(par);
                            else if (q - 1 < A4T) slot_a(par, q - 1);
                            else slot_b(par, q - 1 - A4T);
                        }
                    } else {
                        const int w = q - NLOAD;
                        if (w < A4T) store_a(par ^ 1, w);
                        else store_b(par ^ 1, w - A4T);
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        if (mode > 0) __syncthreads();
    };
    using P0 = std::integral_constant<int, 0>;
    using P1 = std::integral_constant<int, 1>;
    using M2 = std::integral_constant<int, 2>;
    int step = 0;
    for (; step + 3 < nsteps; step += 2) {
        do_step(P0{}, M2{});
        do_step(P1{}, M2{});
    }
    const int rest = nsteps - step;
    if (rest == 3) {
        do_step(P0{}, M2{});
        do_step(P1{}, P1{});
        do_step(P0{}, P0{});
    } else if (rest == 2) {
        do_step(P0{}, P1{});
        do_step(P1{}, P0{});
    } else if (rest == 1) {
        do_step(P0{}, P0{});
    }

    const int plane = p.OH * p.OW;
#pragma unroll
    for (int jn = 0; jn < TN; ++jn) {
        const int col = n0 + (wn * TN + jn) * 32 + l32;
        if (col >= p.ncols) continue;
        const int n = (int)fastdiv((uint32_t)col, p.div_plane);
        const int rem = col - n * plane;
        if (p.epi_on && p.ksplit == 1)            // split sums get it in reduce_split_outputs
            epi_tile<TM, TN>(p.epi, acc, jn, m0 + wm * TM * 32 + half * 4, p.M, plane,
                             (int64_t)n * p.epi.mask_bs + rem);
        if (p.ksplit == 1 && p.out_bf16) {
            unsigned short *out = reinterpret_cast<unsigned short *>(p.dst) + (size_t)n * p.dst_bs + rem;
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                const int row0 = m0 + (wm * TM + i) * 32 + half * 4;
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int row = row0 + (v >> 2) * 8 + (v & 3);
                    if (row < p.M) out[(size_t)row * plane] = bf16_round(acc[i][jn][v]);
                }
            }
            continue;
        }
        float *out = p.ksplit > 1 ? p.part + ((size_t)ks * (p.ncols / plane) + n) * ((size_t)p.M * plane) + rem
                                  : p.dst + (size_t)n * p.dst_bs + rem;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int row0 = m0 + (wm * TM + i) * 32 + half * 4;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = row0 + (v >> 2) * 8 + (v & 3);
                if (row < p.M) out[(size_t)row * plane] = acc[i][jn][v];
            }
        }
    }
}

// NCHW bf16 (samples src_bs elements apart) -> dst[n][c / 16][h*w][16]: the 16 channels of a block at one
// position become 32 contiguous bytes.  One thread per (n, block, position); lanes run along positions.
__global__ void block_channels_bf16(const unsigned short *__restrict__ src, u32x4 *__restrict__ dst, int N, int C,
                                    int HW, int64_t src_bs, FastDiv div_hw)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t total = (int64_t)N * (C / 16) * HW;
    if (i >= total) return;
    const uint32_t nb = fastdiv((uint32_t)i, div_hw);           // n * (C/16) + block
    const int pos = (int)((uint32_t)i - nb * (uint32_t)HW);
    const uint32_t n = nb / (uint32_t)(C / 16), cb = nb - n * (uint32_t)(C / 16);
    const unsigned short *s = src + n * src_bs + (int64_t)cb * 16 * HW + pos;
    unsigned short v[16];
#pragma unroll
    for (int k = 0; k < 16; ++k) v[k] = s[(int64_t)k * HW];
    u32x4 lo, hi;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        lo[k] = (unsigned)v[2 * k] | ((unsigned)v[2 * k + 1] << 16);
        hi[k] = (unsigned)v[8 + 2 * k] | ((unsigned)v[8 + 2 * k + 1] << 16);
    }
    dst[2 * i] = lo;
    dst[2 * i + 1] = hi;
}

// bf16 filters for colgemm_bf16_kernel: wt[((cb*R + r)*S + s)][Mpad][kc]
__global__ void relayout_filters_cblk_bf16(const unsigned short *__restrict__ w, unsigned short *__restrict__ wt,
                                           int M, int Mpad, int cblocks, int RS, int C, int transposed, int kc)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int64_t total = (int64_t)cblocks * RS * Mpad * kc;
    if (i >= total) return;
    int e = (int)(i % kc);
    int64_t t = i / kc;
    int m = (int)(t % Mpad);
    t /= Mpad;
    int rs = (int)(t % RS);
    int cb = (int)(t / RS);
    int ch = cb * kc + e;
    unsigned short v = 0;
    if (m < M) v = transposed ? w[((int64_t)ch * C + m) * RS + rs] : w[((int64_t)m * C + ch) * RS + rs];
    wt[i] = v;
}

// out[n][i] = part[0][n][i] + part[1][n][i] + ...  (fixed order), i over one sample's M*OH*OW outputs
// and the epilogue applied to the sum when epi_on
template <typename T>
__global__ void reduce_split_outputs(const float *__restrict__ part, T *__restrict__ dst, int nsplit,
                                     int per_sample, int N, int dst_bs, FastDiv div_sample, int epi_on, Epilogue epi,
                                     FastDiv div_plane)
{
    const int total = N * per_sample;
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < total; i += gridDim.x * blockDim.x) {
        float v = part[i];
        for (int k = 1; k < nsplit; ++k) v += part[(size_t)k * total + i];
        const int n = (int)fastdiv((uint32_t)i, div_sample);
        const int r = i - n * per_sample;
        if (epi_on) v = epi_apply(epi, v, (int)fastdiv((uint32_t)r, div_plane), (int64_t)n * epi.mask_bs + r);
        st_elem(dst, (int64_t)n * dst_bs + r, v);
    }
}

// Filters for colgemm_fast_kernel: wt[((cb*R + r)*S + s)][Mpad][kc], element e = channel cb*kc+e.
//   transposed = 0: row m = filter k, channel = input channel c   (forward)
//   transposed = 1: row m = input channel c, channel = filter k   (backward-data)
//   groups > 1: the filters of column g start w_gs floats after those of column g - 1; the copies are consecutive
__global__ void relayout_filters_cblk(const float *__restrict__ w, float *__restrict__ wt, int M, int Mpad,
                                      int cblocks, int RS, int C, int transposed, int kc, int groups, int64_t w_gs)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t per = (int64_t)cblocks * RS * Mpad * kc;
    if (i >= per * groups) return;
    const int64_t gcol = i / per;
    w += gcol * w_gs;
    wt += gcol * per;
    i -= gcol * per;
    int e = (int)(i % kc);
    int64_t t = i / kc;
    int m = (int)(t % Mpad);
    t /= Mpad;
    int rs = (int)(t % RS);
    int cb = (int)(t / RS);
    int ch = cb * kc + e;
    float v = 0.f;
    if (m < M) v = transposed ? w[((int64_t)ch * C + m) * RS + rs] : w[((int64_t)m * C + ch) * RS + rs];
    wt[i] = v;
}

// ---------------------------------------------------------------------------
// Forward pass for layers with few input channels (the 11x11 stride-4 first
// layer: C = 3).  A work-group owns 128 consecutive output positions of ONE
// image and stages every input row those positions read -- zero padding
// included -- in LDS once, with coalesced row loads.  The im2col operand is then
// read from that patch: element (g = (c, r, s), position (p, q)) sits at
//   patch[(c*NR + (p - p0)*stride + r) * WP + q*stride + s],
// i.e. a per-lane position offset plus a per-g offset from a small LDS table.
// No gathers from global memory, no padding tests in the loop.  Filters stream
// through LDS 16 deep as in the other kernels.  One wave = TM x 1 tiles of 32x32.
// ---------------------------------------------------------------------------
struct PatchArgs {
    const float *At;      // filters [chunk][Mpad][16], g in (c, r, s) order, zero padded
    const void *x;        // fp32 or bfloat16 (the kernel's TI)
    void *y;              // fp32 or bfloat16 (the kernel's TO)
    int M, Mpad, nchunks;
    int C, H, W, R, S, stride, pad;
    int P, Q, PQ;
    int NR, WP;           // staged rows per channel, LDS row pitch (W + 2*pad rounded up)
    int Kg, Kgpad;
    int x_bs, y_bs;
    int mtiles, jtiles;   // row tiles, position tiles per image
    int ntiles, tiles_per_xcd;
    FastDiv div_q, div_rs, div_s, div_mj, div_m, div_wp, div_nr;
};

template <int TM, typename TI, typename TO>
__global__ __launch_bounds__(kThreads) void colgemm_patch_kernel(const PatchArgs p)
{
    constexpr int BM = TM * 32, BN = 128;
    constexpr int A4 = BM * 4;
    constexpr int A4T = (A4 + kThreads - 1) / kThreads;
    extern __shared__ __attribute__((aligned(16))) float lds_fast[];
    float *const As0 = lds_fast;                               // 2 x BM x kPitch
    int *const koff = reinterpret_cast<int *>(lds_fast + 2 * BM * kPitch);   // Kgpad
    float *const patch = lds_fast + 2 * BM * kPitch + p.Kgpad; // C x NR x WP

    const int bid = blockIdx.x;
    const int idx = bid >> 3;
    const int tile = (bid & 7) * p.tiles_per_xcd + idx;
    if (idx >= p.tiles_per_xcd || tile >= p.ntiles) return;
    // tile -> (image n, position tile jt, row tile mt), row tiles fastest
    const int n = (int)fastdiv((uint32_t)tile, p.div_mj);
    const int rem = tile - n * (p.mtiles * p.jtiles);
    const int jt = (int)fastdiv((uint32_t)rem, p.div_m);
    const int mt = rem - jt * p.mtiles;
    const int m0 = mt * BM, j0 = jt * BN;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = uniform(tid >> 6);
    const int l32 = lane & 31, half = lane >> 5;

    const int p0 = (int)fastdiv((uint32_t)j0, p.div_q);
    const int h0 = p0 * p.stride - p.pad;                      // image row of staged row 0

    // --- stage the patch: row (c, i) <- x[n][c][h0 + i][:], zero outside the image
    {
        // 32 independent loads in flight per thread and batch (the first layer's patch is ~60 values per thread)
        const TI *xn = static_cast<const TI *>(p.x) + (size_t)n * p.x_bs;
        const int total = p.C * p.NR * p.WP;
        for (int e0 = tid; e0 < total; e0 += kThreads * 32) {
            float tmp[32];
#pragma unroll
            for (int u = 0; u < 32; ++u) {
                const int e = e0 + u * kThreads;
                const int ee = e < total ? e : 0;
                const int row = (int)fastdiv((uint32_t)ee, p.div_wp);
                const int v = ee - row * p.WP;
                const int c = (int)fastdiv((uint32_t)row, p.div_nr);
                const int h = h0 + row - c * p.NR, w = v - p.pad;
                const bool ok = ((unsigned)h < (unsigned)p.H) & ((unsigned)w < (unsigned)p.W);
                const float val = ld_elem(xn, ok ? (c * p.H + h) * p.W + w : 0);
                tmp[u] = ok ? val : 0.f;
            }
#pragma unroll
            for (int u = 0; u < 32; ++u) {
                const int e = e0 + u * kThreads;
                if (e < total) patch[e] = tmp[u];
            }
        }
        // per-g offset table; padded g (zero filter) may point anywhere inside the patch
        for (int g = tid; g < p.Kgpad; g += kThreads) {
            int off = 0;
            if (g < p.Kg) {
                const int c = (int)fastdiv((uint32_t)g, p.div_rs);
                const int rs = g - c * (p.R * p.S);
                const int r = (int)fastdiv((uint32_t)rs, p.div_s);
                off = (c * p.NR + r) * p.WP + (rs - r * p.S);
            }
            koff[g] = off;
        }
    }

    // this lane's output position and its offset into the patch
    const int j = j0 + wave * 32 + l32;
    const bool jok = j < p.PQ;
    int colbase;
    {
        const int jj = jok ? j : j0;
        const int pp = (int)fastdiv((uint32_t)jj, p.div_q);
        const int qq = jj - pp * p.Q;
        colbase = (pp - p0) * p.stride * p.WP + qq * p.stride;
    }

    // filter slices: register set t & 1 and LDS buffer t & 1 hold step t; loads run two steps ahead and the LDS
    // writes of the next step sit between the matrix instructions (see colgemm_fast_kernel)
    f32x4 areg[2][A4T];
    const f32x4 *a_ptr = reinterpret_cast<const f32x4 *>(p.At + (size_t)m0 * kChunk) + tid;
    const size_t a_step = (size_t)p.Mpad * (kChunk / 4);
    auto slot_a = [&](int set, int i) {
        if (A4 % kThreads == 0 || tid + i * kThreads < A4) areg[set][i] = a_ptr[i * kThreads];
        if (i == A4T - 1) a_ptr += a_step;
    };
    auto store_a = [&](int set, int i) {
        float *As = As0 + set * BM * kPitch;
        const int q = tid + i * kThreads;
        if (A4 % kThreads == 0 || q < A4) *reinterpret_cast<f32x4 *>(&As[(q >> 2) * kPitch + (q & 3) * 4]) = areg[set][i];
    };

    f32x16 acc[TM];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;

#pragma unroll
    for (int i = 0; i < A4T; ++i) slot_a(0, i);
#pragma unroll
    for (int i = 0; i < A4T; ++i) store_a(0, i);
    if (p.nchunks > 1) {
#pragma unroll
        for (int i = 0; i < A4T; ++i) slot_a(1, i);
    }
    __syncthreads();
    const int a_frag = l32 * kPitch + half * 8;
    // The im2col values do not depend on the filter staging, so those of step+1 are
    // read from the patch while step's matrix instructions run.
    float bv[8];
    auto read_b = [&](int step) {
        const int4 k0 = *reinterpret_cast<const int4 *>(&koff[step * kChunk + half * 8]);
        const int4 k1 = *reinterpret_cast<const int4 *>(&koff[step * kChunk + half * 8 + 4]);
        bv[0] = patch[colbase + k0.x]; bv[1] = patch[colbase + k0.y];
        bv[2] = patch[colbase + k0.z]; bv[3] = patch[colbase + k0.w];
        bv[4] = patch[colbase + k1.x]; bv[5] = patch[colbase + k1.y];
        bv[6] = patch[colbase + k1.z]; bv[7] = patch[colbase + k1.w];
    };
    read_b(0);
    // mode 2: filter loads of step + 2 and stores of step + 1; 1: stores only; 0: neither (par, mode compile-time)
    auto do_step = [&](auto par_c, auto mode_c, int step) {
        constexpr int par = decltype(par_c)::value, mode = decltype(mode_c)::value;
        const float *As = As0 + par * BM * kPitch;
        f32x4 fa[TM][2];
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const f32x4 *q = reinterpret_cast<const f32x4 *>(&As[a_frag + i * 32 * kPitch]);
            fa[i][0] = q[0]; fa[i][1] = q[1];
        }
        float bc[8];
#pragma unroll
        for (int t = 0; t < 8; ++t) bc[t] = bv[t];
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int t = 0; t < 8; ++t) {
#pragma unroll
            for (int i = 0; i < TM; ++i)
                acc[i] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[i][t >> 2][t & 3], bc[t], acc[i], 0, 0, 0);
            if (mode > 0) {
                __builtin_amdgcn_sched_barrier(0);
                if (mode == 2 && t < A4T) slot_a(par, t);
                if (t == 3) read_b(step + 1);
                if (t >= 4 && t - 4 < A4T) store_a(par ^ 1, t - 4);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        if (mode > 0) __syncthreads();
    };
    static_assert(A4T <= 4, "filter slots fit the eight reduction pairs of a step");
    using P0 = std::integral_constant<int, 0>;
    using P1 = std::integral_constant<int, 1>;
    using M2 = std::integral_constant<int, 2>;
    int step = 0;
    for (; step + 3 < p.nchunks; step += 2) {
        do_step(P0{}, M2{}, step);
        do_step(P1{}, M2{}, step + 1);
    }
    const int rest = p.nchunks - step;
    if (rest == 3) {
        do_step(P0{}, M2{}, step);
        do_step(P1{}, P1{}, step + 1);
        do_step(P0{}, P0{}, step + 2);
    } else if (rest == 2) {
        do_step(P0{}, P1{}, step);
        do_step(P1{}, P0{}, step + 1);
    } else if (rest == 1) {
        do_step(P0{}, P0{}, step);
    }

    if (!jok) return;
    TO *out = static_cast<TO *>(p.y) + (size_t)n * p.y_bs + j;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int row0 = m0 + i * 32 + half * 4;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int row = row0 + (v >> 2) * 8 + (v & 3);
            if (row < p.M) st_elem(out, (int64_t)row * p.PQ, acc[i][v]);
        }
    }
}

// ---------------------------------------------------------------------------
// Backward-filter: dw[k][g] = sum_j dy[k][j] * im2col(x)[g][j],  j = (n, p, q)
// ---------------------------------------------------------------------------
struct WgradArgs {
    const void *dy;       // fp32 or bfloat16 (the kernel's TI), both inputs alike
    const void *x;
    const int4 *tab;      // forward-style tap table over g = (c, r, s)
    float *out;           // dw, or partial sums [split][K][CRS]
    int K, CRS;
    int P, Q, H, W, stride, pad;
    int dy_bs, x_bs;
    int J;                // N*P*Q
    int chunks_per_split;
    int mtiles, ntiles;
    int units, units_per_xcd;   // units = tiles * splits; the grid is 8 * units_per_xcd
    FastDiv div_plane, div_q;
};

template <int TM, int TN, int WM, int WN, typename TI>
__global__ __launch_bounds__(kThreads) void wgrad_kernel(const WgradArgs p)
{
    constexpr int BM = TM * WM * 32, BN = TN * WN * 32;
    constexpr int RA = BM / 16, RB = BN / 16;    // rows per thread per step
    constexpr int EB = (int)sizeof(TI);          // bytes per input element
    static_assert(WM * WN == 4, "four waves per work-group");

    __shared__ __attribute__((aligned(16))) float As[2][BM * kPitch];
    __shared__ __attribute__((aligned(16))) float Bs[2][BN * kPitch];

    // Work-groups are dealt round-robin to the 8 XCDs; each XCD takes a contiguous eighth of the (split, tile)
    // list, so the tiles of one split -- which read the same range of dy and overlapping rows of x -- run on
    // one XCD at the same time and share its L2.
    const int tiles = p.mtiles * p.ntiles;
    const int unit = (blockIdx.x & 7) * p.units_per_xcd + (blockIdx.x >> 3);
    if ((int)(blockIdx.x >> 3) >= p.units_per_xcd || unit >= p.units) return;
    const int split = unit / tiles;
    const int tile = unit - split * tiles;
    const int mt = tile % p.mtiles, nt = tile / p.mtiles;
    const int m0 = mt * BM, n0 = nt * BN;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = uniform(tid >> 6);
    const int wm = wave / WN, wn = wave % WN;

    // loader role: reduction position jj of the step, rows g, g+16, ...
    const int jj = tid & 15, g = tid >> 4;
    const int PQ = p.P * p.Q;

    int boff[RB], bdr[RB], bds[RB];
#pragma unroll
    for (int i = 0; i < RB; ++i) {
        const int4 tap = p.tab[n0 + g + 16 * i];     // table is padded past CRS with failing taps
        boff[i] = tap.x / 4 * EB; bdr[i] = tap.y; bds[i] = tap.z;     // the table holds byte offsets of fp32 elements
    }

    const int jbeg = split * p.chunks_per_split * kChunk;
    int jend = jbeg + p.chunks_per_split * kChunk;
    if (jend > p.J) jend = p.J;
    const int nsteps = (jend - jbeg + kChunk - 1) / kChunk;

    // register set t & 1 and LDS buffer t & 1 hold step t; loads run two steps ahead and the LDS writes of the
    // next step sit between the matrix instructions of the current one (see colgemm_fast_kernel)
    TI areg[2][RA], breg[2][RB];                 // as loaded; widened when they are written to LDS
    bool aok[2][RA], bok[2][RB];
    const char *dy_bytes = reinterpret_cast<const char *>(p.dy);
    const char *x_bytes = reinterpret_cast<const char *>(p.x);
    int abase = 0, bbase = 0, hb = 0, wb = 0, jnext = jbeg + jj;
    bool jok = false;

    auto slot_pos = [&]() {          // where this thread's reduction position sits
        jok = jnext < jend;
        const int js = jok ? jnext : jbeg;
        const int n = (int)fastdiv((uint32_t)js, p.div_plane);
        const int pq = js - n * PQ;
        const int pp = (int)fastdiv((uint32_t)pq, p.div_q);
        const int qq = pq - pp * p.Q;
        const int hb0 = pp * p.stride - p.pad;
        wb = qq * p.stride - p.pad;
        abase = EB * (n * p.dy_bs + pq);                 // bytes
        bbase = EB * (n * p.x_bs + hb0 * p.W + wb);
        hb = jok ? hb0 : kInvalidTap;
        jnext += kChunk;
    };
    auto slot_a = [&](int set, int i) {
        const int k = m0 + g + 16 * i;
        const bool ok = jok & (k < p.K);
        areg[set][i] = *reinterpret_cast<const TI *>(dy_bytes + (uint32_t)(ok ? abase + EB * k * PQ : 0));
        aok[set][i] = ok;
    };
    auto slot_b = [&](int set, int i) {
        const int hh = hb + bdr[i], ww = wb + bds[i];
        const bool ok = ((unsigned)hh < (unsigned)p.H) & ((unsigned)ww < (unsigned)p.W);
        breg[set][i] = *reinterpret_cast<const TI *>(x_bytes + (uint32_t)(ok ? bbase + boff[i] : 0));
        bok[set][i] = ok;
    };
    auto load_step = [&](int set) {
        slot_pos();
#pragma unroll
        for (int i = 0; i < RA; ++i) slot_a(set, i);
#pragma unroll
        for (int i = 0; i < RB; ++i) slot_b(set, i);
    };
    auto store_a = [&](int set, int i) {
        As[set][(g + 16 * i) * kPitch + jj] = aok[set][i] ? widen_elem(areg[set][i]) : 0.f;
    };
    auto store_b = [&](int set, int i) {
        Bs[set][(g + 16 * i) * kPitch + jj] = bok[set][i] ? widen_elem(breg[set][i]) : 0.f;
    };
    auto store_step = [&](int set) {
#pragma unroll
        for (int i = 0; i < RA; ++i) store_a(set, i);
#pragma unroll
        for (int i = 0; i < RB; ++i) store_b(set, i);
    };

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int jn = 0; jn < TN; ++jn)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][jn][v] = 0.f;

    const int l32 = lane & 31, half = lane >> 5;
    const int a_frag = (wm * TM * 32 + l32) * kPitch + half * 8;
    const int b_frag = (wn * TN * 32 + l32) * kPitch + half * 8;
    constexpr int NMMA = 8 * TM * TN;
    constexpr int NLOAD = 1 + RA + RB, NSTORE = RA + RB;
    constexpr int SPM = (NLOAD + NSTORE + NMMA - 3) / (NMMA - 2);

    if (nsteps > 0) {
        load_step(0);
        store_step(0);
        if (nsteps > 1) load_step(1);
    }
    __syncthreads();
    // mode 2: loads of step + 2 and stores of step + 1; 1: stores only; 0: neither (par, mode compile-time)
    auto do_step = [&](auto par_c, auto mode_c) {
        constexpr int par = decltype(par_c)::value, mode = decltype(mode_c)::value;
        f32x4 fa[TM][2], fb[TN][2];
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const f32x4 *q = reinterpret_cast<const f32x4 *>(&As[par][a_frag + i * 32 * kPitch]);
            fa[i][0] = q[0]; fa[i][1] = q[1];
        }
#pragma unroll
        for (int jn = 0; jn < TN; ++jn) {
            const f32x4 *q = reinterpret_cast<const f32x4 *>(&Bs[par][b_frag + jn * 32 * kPitch]);
            fb[jn][0] = q[0]; fb[jn][1] = q[1];
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int m = 0; m < NMMA; ++m) {
            const int t = m / (TM * TN), i = (m / TN) % TM, jn = m % TN;
            acc[i][jn] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[i][t >> 2][t & 3], fb[jn][t >> 2][t & 3],
                                                              acc[i][jn], 0, 0, 0);
            if (mode > 0 && m * SPM < NLOAD + NSTORE) {
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int q = m * SPM; q < (m + 1) * SPM && q < NLOAD + NSTORE; ++q) {
                    if (q < NLOAD) {
                        if (mode == 2) {
                            if (q == 0) slot_pos();
                            else if (q - 1 < RA) slot_a(par, q - 1);
                            else slot_b(par, q - 1 - RA);
                        }
                    } else {
                        const int w = q - NLOAD;
                        if (w < RA) store_a(par ^ 1, w);
                        else store_b(par ^ 1, w - RA);
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        if (mode > 0) __syncthreads();
    };
    using P0 = std::integral_constant<int, 0>;
    using P1 = std::integral_constant<int, 1>;
    using M2 = std::integral_constant<int, 2>;
    int step = 0;
    for (; step + 3 < nsteps; step += 2) {
        do_step(P0{}, M2{});
        do_step(P1{}, M2{});
    }
    const int rest = nsteps - step;
    if (rest == 3) {
        do_step(P0{}, M2{});
        do_step(P1{}, P1{});
        do_step(P0{}, P0{});
    } else if (rest == 2) {
        do_step(P0{}, P1{});
        do_step(P1{}, P0{});
    } else if (rest == 1) {
        do_step(P0{}, P0{});
    }

    float *out = p.out + (size_t)split * p.K * p.CRS;
#pragma unroll
    for (int jn = 0; jn < TN; ++jn) {
        const int col = n0 + (wn * TN + jn) * 32 + l32;
        if (col >= p.CRS) continue;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int row0 = m0 + (wm * TM + i) * 32 + half * 4;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = row0 + (v >> 2) * 8 + (v & 3);
                if (row < p.K) out[(size_t)row * p.CRS + col] = acc[i][jn][v];
            }
        }
    }
}

// ---------------------------------------------------------------------------
// Backward-filter when C is a multiple of 16.  The GEMM columns are taken in
// (r, s, c) order, c fastest, so the rows a thread stages (a block of BN/16
// consecutive columns) are consecutive channels of ONE filter tap: one padding
// test and one base address per step, channel stride between its loads -- the
// same economy as colgemm_fast_kernel.  Partial sums land in the workspace as
// [split][K][R*S*C]; finish_wgrad adds the splits in order and writes KCRS.
// ---------------------------------------------------------------------------
struct WgradFastArgs {
    const float *dy;
    const float *x;
    float *part;          // [nsplit][K][ncols], columns in (r, s, c) order
    int K, C, S, ncols;   // ncols = R*S*C
    int P, Q, H, W, stride, pad;
    int dy_bs, x_bs;
    int J, chunks_per_split;
    int mtiles, ntiles, nunits, units_per_xcd;
    int x_plane_bytes, y_plane_bytes;
    // columns of a grouped layer in one launch (fp32 kernel): nunits = tiles * nsplit * groups; column g reads
    // dy + g * dy_gs and x + g * x_gs and writes part + g * part_gs (floats)
    int nsplit, groups;
    int64_t dy_gs, x_gs, part_gs;
    FastDiv div_plane, div_q, div_c;
};

template <int TM, int TN, int WM, int WN>
__global__ __launch_bounds__(kThreads) void wgrad_fast_kernel(const WgradFastArgs p)
{
    constexpr int BM = TM * WM * 32, BN = TN * WN * 32;
    constexpr int RA = BM / 16, RB = BN / 16;
    static_assert(WM * WN == 4, "four waves per work-group");

    __shared__ __attribute__((aligned(16))) float As[2][BM * kPitch];
    __shared__ __attribute__((aligned(16))) float Bs[2][BN * kPitch];

    const int bid = blockIdx.x;
    const int idx = bid >> 3;
    const int unit = (bid & 7) * p.units_per_xcd + idx;
    if (idx >= p.units_per_xcd || unit >= p.nunits) return;
    const int tiles = p.mtiles * p.ntiles;
    const int grp_col = unit / (tiles * p.nsplit);              // column of a grouped layer
    const int unit_c = unit - grp_col * (tiles * p.nsplit);
    const int split = unit_c / tiles;
    const int tile = unit_c - split * tiles;
    const int mt = tile % p.mtiles, nt = tile / p.mtiles;
    const int m0 = mt * BM, n0 = nt * BN;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = uniform(tid >> 6);
    const int wm = wave / WN, wn = wave % WN;
    const int jj = tid & 15, g = tid >> 4;
    const int PQ = p.P * p.Q;

    // A rows (filters k): a block of RA consecutive rows; rows past K are clamped
    // for the address and zeroed by a_rows
    const int arow0 = m0 + g * RA;
    const int a_rows = min(max(p.K - arow0, 0), RA);
    int a_off[RA];
#pragma unroll
    for (int i = 0; i < RA; ++i) a_off[i] = min(arow0 + i, p.K - 1) * p.y_plane_bytes;

    // B rows (columns of dw): RB consecutive channels of one tap
    const int col0 = n0 + g * RB;
    const bool col_ok = col0 < p.ncols;
    int tap_r, tap_s, b_off;
    {
        const int cc = col_ok ? col0 : 0;
        const int rs = (int)fastdiv((uint32_t)cc, p.div_c);
        const int c0 = cc - rs * p.C;
        tap_r = rs / p.S;
        tap_s = rs - tap_r * p.S;
        b_off = c0 * p.x_plane_bytes + 4 * (tap_r * p.W + tap_s);
    }

    const int jbeg = split * p.chunks_per_split * kChunk;
    const int jend = min(jbeg + p.chunks_per_split * kChunk, p.J);
    const int nsteps = (jend - jbeg + kChunk - 1) / kChunk;

    const char *dy_bytes = reinterpret_cast<const char *>(p.dy + (size_t)grp_col * p.dy_gs);
    const char *x_bytes = reinterpret_cast<const char *>(p.x + (size_t)grp_col * p.x_gs);
    // Register set t & 1 and LDS buffer t & 1 hold step t; loads run two steps ahead and the LDS writes of the
    // next step sit between the matrix instructions of the current one (see colgemm_fast_kernel).
    float areg[2][RA], breg[2][RB];
    int a_lim[2] = {0, 0}, abase = 0, bbase = 0, jnext = jbeg + jj;
    bool bok[2] = {false, false};

    auto slot_pos = [&](int set) {   // where this thread's reduction position sits
        const bool jok = jnext < jend;
        const int js = jok ? jnext : jbeg;
        const int n = (int)fastdiv((uint32_t)js, p.div_plane);
        const int pq = js - n * PQ;
        const int pp = (int)fastdiv((uint32_t)pq, p.div_q);
        const int qq = pq - pp * p.Q;
        const int hb = pp * p.stride - p.pad, wb = qq * p.stride - p.pad;
        a_lim[set] = jok ? a_rows : 0;
        abase = 4 * (n * p.dy_bs + pq);
        bok[set] = jok & col_ok & ((unsigned)(hb + tap_r) < (unsigned)p.H) & ((unsigned)(wb + tap_s) < (unsigned)p.W);
        bbase = bok[set] ? 4 * (n * p.x_bs + hb * p.W + wb) + b_off : 0;
        jnext += kChunk;
    };
    auto slot_a = [&](int set, int i) {
        areg[set][i] = *reinterpret_cast<const float *>(dy_bytes + (uint32_t)(abase + a_off[i]));
    };
    auto slot_b = [&](int set, int i) {
        breg[set][i] = *reinterpret_cast<const float *>(x_bytes + (uint32_t)(bbase + i * p.x_plane_bytes));
    };
    auto load_step = [&](int set) {
        slot_pos(set);
#pragma unroll
        for (int i = 0; i < RA; ++i) slot_a(set, i);
#pragma unroll
        for (int i = 0; i < RB; ++i) slot_b(set, i);
    };
    auto store_a = [&](int set, int i) {
        As[set][(g * RA + i) * kPitch + jj] = i < a_lim[set] ? areg[set][i] : 0.f;
    };
    auto store_b = [&](int set, int i) {
        Bs[set][(g * RB + i) * kPitch + jj] = bok[set] ? breg[set][i] : 0.f;
    };
    auto store_step = [&](int set) {
#pragma unroll
        for (int i = 0; i < RA; ++i) store_a(set, i);
#pragma unroll
        for (int i = 0; i < RB; ++i) store_b(set, i);
    };

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int jn = 0; jn < TN; ++jn)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][jn][v] = 0.f;

    const int l32 = lane & 31, half = lane >> 5;
    const int a_frag = (wm * TM * 32 + l32) * kPitch + half * 8;
    const int b_frag = (wn * TN * 32 + l32) * kPitch + half * 8;
    constexpr int NMMA = 8 * TM * TN;
    constexpr int NLOAD = 1 + RA + RB, NSTORE = RA + RB;
    constexpr int SPM = (NLOAD + NSTORE + NMMA - 3) / (NMMA - 2);

    if (nsteps > 0) {
        load_step(0);
        store_step(0);
        if (nsteps > 1) load_step(1);
    }
    __syncthreads();
    // mode 2: loads of step + 2 and stores of step + 1; 1: stores only; 0: neither (par, mode compile-time)
    auto do_step = [&](auto par_c, auto mode_c) {
        constexpr int par = decltype(par_c)::value, mode = decltype(mode_c)::value;
        f32x4 fa[TM][2], fb[TN][2];
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const f32x4 *q = reinterpret_cast<const f32x4 *>(&As[par][a_frag + i * 32 * kPitch]);
            fa[i][0] = q[0]; fa[i][1] = q[1];
        }
#pragma unroll
        for (int jn = 0; jn < TN; ++jn) {
            const f32x4 *q = reinterpret_cast<const f32x4 *>(&Bs[par][b_frag + jn * 32 * kPitch]);
            fb[jn][0] = q[0]; fb[jn][1] = q[1];
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int m = 0; m < NMMA; ++m) {
            const int t = m / (TM * TN), i = (m / TN) % TM, jn = m % TN;
            acc[i][jn] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[i][t >> 2][t & 3], fb[jn][t >> 2][t & 3],
                                                              acc[i][jn], 0, 0, 0);
            if (mode > 0 && m * SPM < NLOAD + NSTORE) {
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int q = m * SPM; q < (m + 1) * SPM && q < NLOAD + NSTORE; ++q) {
                    if (q < NLOAD) {
                        if (mode == 2) {
                            if (q == 0) slot_pos(par);
                            else if (q - 1 < RA) slot_a(par, q - 1);
                            else slot_b(par, q - 1 - RA);
                        }
                    } else {
                        const int w = q - NLOAD;
                        if (w < RA) store_a(par ^ 1, w);
                        else store_b(par ^ 1, w - RA);
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        if (mode > 0) __syncthreads();
    };
    using P0 = std::integral_constant<int, 0>;
    using P1 = std::integral_constant<int, 1>;
    using M2 = std::integral_constant<int, 2>;
    int step = 0;
    for (; step + 3 < nsteps; step += 2) {
        do_step(P0{}, M2{});
        do_step(P1{}, M2{});
    }
    const int rest = nsteps - step;                 // up to 3 steps left, the first in buffer 0
    if (rest == 3) {
        do_step(P0{}, M2{});
        do_step(P1{}, P1{});
        do_step(P0{}, P0{});
    } else if (rest == 2) {
        do_step(P0{}, P1{});
        do_step(P1{}, P0{});
    } else if (rest == 1) {
        do_step(P0{}, P0{});
    }

    float *out = p.part + (size_t)grp_col * p.part_gs + (size_t)split * p.K * p.ncols;
#pragma unroll
    for (int jn = 0; jn < TN; ++jn) {
        const int col = n0 + (wn * TN + jn) * 32 + l32;
        if (col >= p.ncols) continue;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int row0 = m0 + (wm * TM + i) * 32 + half * 4;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = row0 + (v >> 2) * 8 + (v & 3);
                if (row < p.K) out[(size_t)row * p.ncols + col] = acc[i][jn][v];
            }
        }
    }
}

// ---------------------------------------------------------------------------
// Backward-filter with bf16 inputs on v_mfma_f32_32x32x16_bf16.  Same column
// order and split scheme as wgrad_fast_kernel; a step covers 64 reduction
// positions.  A thread stages a PAIR of adjacent positions for 16 rows of dy and
// 16 channels of one tap of x (2-byte loads, lanes along positions), packs each
// pair into one dword and writes it to the [row][64 positions] LDS tiles, from
// which every MFMA operand (8 consecutive positions of a row) is one b128 read.
// ---------------------------------------------------------------------------
template <int TM, int TN, int WM, int WN, int KJ>
__global__ __launch_bounds__(kThreads) void wgrad_bf16_kernel(const WgradFastArgs p)
{
    constexpr int BM = TM * WM * 32, BN = TN * WN * 32;
    constexpr int GROUPS = 2 * kThreads / KJ;   // row groups: a thread stages BM/GROUPS + BN/GROUPS rows of one position pair
    constexpr int PITCHB = KJ * 2 + 16;
    constexpr int NK = KJ / 16;
    constexpr int RA = BM / GROUPS, RB = BN / GROUPS;
    static_assert(WM * WN == 4, "four waves per work-group");

    extern __shared__ __attribute__((aligned(16))) float lds_fast[];
    char *const As0 = reinterpret_cast<char *>(lds_fast);
    char *const Bs0 = As0 + 2 * BM * PITCHB;

    const int bid = blockIdx.x;
    const int idx = bid >> 3;
    const int unit = (bid & 7) * p.units_per_xcd + idx;
    if (idx >= p.units_per_xcd || unit >= p.nunits) return;
    const int tiles = p.mtiles * p.ntiles;
    const int split = unit / tiles;
    const int tile = unit - split * tiles;
    const int mt = tile % p.mtiles, nt = tile / p.mtiles;
    const int m0 = mt * BM, n0 = nt * BN;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = uniform(tid >> 6);
    const int wm = wave / WN, wn = wave % WN;
    const int jp = tid % (KJ / 2), g = tid / (KJ / 2);
    const int PQ = p.P * p.Q;

    const int arow0 = m0 + g * RA;
    const int a_rows = min(max(p.K - arow0, 0), RA);
    int a_off[RA];
#pragma unroll
    for (int i = 0; i < RA; ++i) a_off[i] = min(arow0 + i, p.K - 1) * p.y_plane_bytes;

    const int col0 = n0 + g * RB;
    const bool col_ok = col0 < p.ncols;
    int tap_r, tap_s, b_off;
    {
        const int cc = col_ok ? col0 : 0;
        const int rs = (int)fastdiv((uint32_t)cc, p.div_c);
        const int c0 = cc - rs * p.C;
        tap_r = rs / p.S;
        tap_s = rs - tap_r * p.S;
        b_off = c0 * p.x_plane_bytes + 2 * (tap_r * p.W + tap_s);
    }

    // chunks_per_split counts 16-position chunks; steps here are KJ positions
    const int steps_per_split = (p.chunks_per_split * 16 + KJ - 1) / KJ;
    const int jbeg = split * steps_per_split * KJ;
    const int jend = min(jbeg + steps_per_split * KJ, p.J);
    const int nsteps = jend > jbeg ? (jend - jbeg + KJ - 1) / KJ : 0;

    const char *dy_bytes = reinterpret_cast<const char *>(p.dy);
    const char *x_bytes = reinterpret_cast<const char *>(p.x);
    unsigned short areg[2][RA], breg[2][RB];
    int a_lim[2] = {0, 0}, abase[2] = {0, 0}, bbase[2] = {0, 0};
    bool bok[2] = {false, false};
    int jnext = jbeg + 2 * jp;

    auto slot_pos = [&]() {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int j = jnext + h;
            const bool jok = j < jend;
            const int js = jok ? j : jbeg;
            const int n = (int)fastdiv((uint32_t)js, p.div_plane);
            const int pq = js - n * PQ;
            const int pp = (int)fastdiv((uint32_t)pq, p.div_q);
            const int qq = pq - pp * p.Q;
            const int hb = pp * p.stride - p.pad, wb = qq * p.stride - p.pad;
            a_lim[h] = jok ? a_rows : 0;
            abase[h] = 2 * (n * p.dy_bs + pq);
            bok[h] = jok & col_ok & ((unsigned)(hb + tap_r) < (unsigned)p.H) & ((unsigned)(wb + tap_s) < (unsigned)p.W);
            bbase[h] = bok[h] ? 2 * (n * p.x_bs + hb * p.W + wb) + b_off : 0;
        }
        jnext += KJ;
    };
    auto slot_a = [&](int q) {       // q = 2*i + h
        const int i = q >> 1, h = q & 1;
        areg[h][i] = *reinterpret_cast<const unsigned short *>(dy_bytes + (uint32_t)(abase[h] + a_off[i]));
    };
    auto slot_b = [&](int q) {
        const int i = q >> 1, h = q & 1;
        breg[h][i] = *reinterpret_cast<const unsigned short *>(x_bytes + (uint32_t)(bbase[h] + i * p.x_plane_bytes));
    };
    auto load_step = [&]() {
        slot_pos();
#pragma unroll
        for (int q = 0; q < 2 * RA; ++q) slot_a(q);
#pragma unroll
        for (int q = 0; q < 2 * RB; ++q) slot_b(q);
    };
    auto store_step = [&](int buf) {
        char *As = As0 + buf * BM * PITCHB, *Bs = Bs0 + buf * BN * PITCHB;
#pragma unroll
        for (int i = 0; i < RA; ++i) {
            const unsigned lo = i < a_lim[0] ? (unsigned)areg[0][i] : 0u;
            const unsigned hi = i < a_lim[1] ? (unsigned)areg[1][i] : 0u;
            *reinterpret_cast<unsigned *>(As + (g * RA + i) * PITCHB + jp * 4) = lo | (hi << 16);
        }
#pragma unroll
        for (int i = 0; i < RB; ++i) {
            const unsigned lo = bok[0] ? (unsigned)breg[0][i] : 0u;
            const unsigned hi = bok[1] ? (unsigned)breg[1][i] : 0u;
            *reinterpret_cast<unsigned *>(Bs + (g * RB + i) * PITCHB + jp * 4) = lo | (hi << 16);
        }
    };

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int jn = 0; jn < TN; ++jn)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][jn][v] = 0.f;

    const int l32 = lane & 31, half = lane >> 5;
    const int a_frag = (wm * TM * 32 + l32) * PITCHB + half * 16;
    const int b_frag = (wn * TN * 32 + l32) * PITCHB + half * 16;
    constexpr int NMMA = NK * TM * TN;
    constexpr int NSLOT = 1 + 2 * RA + 2 * RB;
    constexpr int SPM = (NSLOT + (NMMA > 2 ? NMMA - 2 : 1) - 1) / (NMMA > 2 ? NMMA - 2 : 1);

    if (nsteps > 0) {
        load_step();
        store_step(0);
    }
    __syncthreads();
    for (int step = 0; step < nsteps; ++step) {
        const int buf = step & 1;
        const bool last = step == nsteps - 1;
        const char *As = As0 + buf * BM * PITCHB, *Bs = Bs0 + buf * BN * PITCHB;
        u32x4 fa[TM][NK], fb[TN][NK];
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int t = 0; t < NK; ++t)
                fa[i][t] = *reinterpret_cast<const u32x4 *>(As + a_frag + i * 32 * PITCHB + t * 32);
#pragma unroll
        for (int jn = 0; jn < TN; ++jn)
#pragma unroll
            for (int t = 0; t < NK; ++t)
                fb[jn][t] = *reinterpret_cast<const u32x4 *>(Bs + b_frag + jn * 32 * PITCHB + t * 32);
        __builtin_amdgcn_sched_barrier(0);
        if (!last) {
#pragma unroll
            for (int m = 0; m < NMMA; ++m) {
                const int t = m / (TM * TN), i = (m / TN) % TM, jn = m % TN;
                acc[i][jn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fa[i][t]),
                                                                     __builtin_bit_cast(bf16x8, fb[jn][t]),
                                                                     acc[i][jn], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int q = m * SPM; q < (m + 1) * SPM && q < NSLOT; ++q) {
                    if (q == 0) slot_pos();
                    else if (q - 1 < 2 * RA) slot_a(q - 1);
                    else slot_b(q - 1 - 2 * RA);
                }
                if (m * SPM < NSLOT) __builtin_amdgcn_sched_barrier(0);
            }
            store_step(buf ^ 1);
            __syncthreads();
        } else {
#pragma unroll
            for (int m = 0; m < NMMA; ++m) {
                const int t = m / (TM * TN), i = (m / TN) % TM, jn = m % TN;
                acc[i][jn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fa[i][t]),
                                                                     __builtin_bit_cast(bf16x8, fb[jn][t]),
                                                                     acc[i][jn], 0, 0, 0);
            }
        }
    }

    float *out = p.part + (size_t)split * p.K * p.ncols;
#pragma unroll
    for (int jn = 0; jn < TN; ++jn) {
        const int col = n0 + (wn * TN + jn) * 32 + l32;
        if (col >= p.ncols) continue;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int row0 = m0 + (wm * TM + i) * 32 + half * 4;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = row0 + (v >> 2) * 8 + (v & 3);
                if (row < p.K) out[(size_t)row * p.ncols + col] = acc[i][jn][v];
            }
        }
    }
}

// ---------------------------------------------------------------------------
// Backward-filter with bf16 inputs for stride-1 layers whose output has the
// input's extent (R - 1 = S - 1 = 2 * pad): every MFMA operand (8 consecutive
// reduction positions of a row) is ONE 16-byte global load.
//
// Two packing passes lay the tensors out for that.  With row pitch Wq = W + pad,
//   dyp[k][n][Jy]: dy(n, k, p, q) at j = p*Wq + q, zeros in the pad columns and in
//                  the tail up to Jy (a multiple of 8); rows zero-filled up to a
//                  whole number of 64-position steps;
//   xp[c][n][Jx]:  x(n, c, h, w) at (h + pad)*Wq + (w + pad), zeros elsewhere.
// The input element that dy position j meets under tap (r, s) then sits at
// j + r*Wq + s of the same image: a column that would wrap lands in the pad
// columns of the neighbouring row (one gap serves as right pad of a row and left
// pad of the next), a row out of range in the zero rows above and below.  No
// masks and no per-element addresses are left; positions where dy is zero cost
// (Jy / (P*Q) - 1) extra matrix work, 9 % at 13x13.
// The x loads are 2-byte aligned only (the tap shift is arbitrary).
// Columns in (r, s, c) order, partials [split][K][R*S*C] as in wgrad_fast_kernel.
// ---------------------------------------------------------------------------
struct WgradLinArgs {
    const unsigned short *dyp;
    const unsigned short *xp;
    float *part;
    int K, C, ncols;
    int S, Wq;
    int N, G, Jx;             // G = Jy / 8 groups of 8 positions per image
    int row_a_bytes;          // bytes per dyp row
    int row_x_bytes;          // bytes per xp row (N * Jx * 2)
    int steps, steps_per_split;
    int mtiles, ntiles, nunits, units_per_xcd;
    FastDiv div_c, div_s, div_g;
};

typedef u32x4 u32x4_align2 __attribute__((aligned(2)));

template <int TM, int TN, int WM, int WN>
__global__ __launch_bounds__(kThreads, 2) void wgrad_bf16_lin_kernel(const WgradLinArgs p)
{
    constexpr int BM = TM * WM * 32, BN = TN * WN * 32;
    constexpr int KJ = 64, NK = KJ / 16;
    constexpr int PITCHB = KJ * 2 + 16;
    constexpr int RA = BM / 32, RB = BN / 32;      // 16-byte vectors per thread and step
    static_assert(WM * WN == 4, "four waves per work-group");

    extern __shared__ __attribute__((aligned(16))) float lds_fast[];
    char *const As0 = reinterpret_cast<char *>(lds_fast);
    char *const Bs0 = As0 + 2 * BM * PITCHB;

    const int bid = blockIdx.x;
    const int idx = bid >> 3;
    const int unit = (bid & 7) * p.units_per_xcd + idx;
    if (idx >= p.units_per_xcd || unit >= p.nunits) return;
    const int ntile = p.mtiles * p.ntiles;
    const int split = unit / ntile;
    const int tile = unit - split * ntile;
    const int mt = tile % p.mtiles, nt = tile / p.mtiles;
    const int m0 = mt * BM, n0 = nt * BN;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = uniform(tid >> 6);
    const int wm = wave / WN, wn = wave % WN;
    const int jg = tid & 7, r8 = tid >> 3;         // this thread's group of 8 positions in a step; its row inside 32

    const int step_begin = split * p.steps_per_split;
    const int nsteps = min(p.steps - step_begin, p.steps_per_split);

    uint32_t abase[RA], bbase[RB];
#pragma unroll
    for (int i = 0; i < RA; ++i) abase[i] = (uint32_t)min(m0 + r8 + 32 * i, p.K - 1) * (uint32_t)p.row_a_bytes;
#pragma unroll
    for (int i = 0; i < RB; ++i) {
        int col = n0 + r8 + 32 * i;
        col = col < p.ncols ? col : 0;
        const int rs = (int)fastdiv((uint32_t)col, p.div_c), c = col - rs * p.C;
        const int r = (int)fastdiv((uint32_t)rs, p.div_s), sx = rs - r * p.S;
        bbase[i] = (uint32_t)c * (uint32_t)p.row_x_bytes + 2u * (uint32_t)(r * p.Wq + sx);
    }
    // position of this thread's group: g = step*8 + jg = n*G + gg
    int n, gg;
    {
        const int g = step_begin * 8 + jg;
        n = (int)fastdiv((uint32_t)g, p.div_g);
        gg = g - n * p.G;
    }
    uint32_t aoff = (uint32_t)(step_begin * 8 + jg) * 16u, boff = 0;
    const char *ap = reinterpret_cast<const char *>(p.dyp), *xp = reinterpret_cast<const char *>(p.xp);

    // register set t & 1 and LDS buffer t & 1 hold step t (two-set pipeline of colgemm_fast_kernel)
    u32x4 areg[2][RA], breg[2][RB];
    auto slot_pos = [&]() {
        boff = 2u * (uint32_t)(min(n, p.N - 1) * p.Jx + gg * 8);
        gg += 8;
        const bool wrap = gg >= p.G;
        gg -= wrap ? p.G : 0;
        n += wrap ? 1 : 0;
    };
    auto slot_a = [&](int set, int i) {
        areg[set][i] = *reinterpret_cast<const u32x4 *>(ap + (abase[i] + aoff));
        if (i == RA - 1) aoff += 128u;
    };
    auto slot_b = [&](int set, int i) {
        breg[set][i] = *reinterpret_cast<const u32x4_align2 *>(xp + (bbase[i] + boff));
    };
    auto load_step = [&](int set) {
        slot_pos();
#pragma unroll
        for (int i = 0; i < RA; ++i) slot_a(set, i);
#pragma unroll
        for (int i = 0; i < RB; ++i) slot_b(set, i);
    };
    auto store_a = [&](int set, int i) {
        *reinterpret_cast<u32x4 *>(As0 + set * BM * PITCHB + (r8 + i * 32) * PITCHB + jg * 16) = areg[set][i];
    };
    auto store_b = [&](int set, int i) {
        *reinterpret_cast<u32x4 *>(Bs0 + set * BN * PITCHB + (r8 + i * 32) * PITCHB + jg * 16) = breg[set][i];
    };
    auto store_step = [&](int set) {
#pragma unroll
        for (int i = 0; i < RA; ++i) store_a(set, i);
#pragma unroll
        for (int i = 0; i < RB; ++i) store_b(set, i);
    };

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int jn = 0; jn < TN; ++jn)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][jn][v] = 0.f;

    const int l32 = lane & 31, half = lane >> 5;
    const int a_frag = (wm * TM * 32 + l32) * PITCHB + half * 16;
    const int b_frag = (wn * TN * 32 + l32) * PITCHB + half * 16;
    constexpr int NMMA = NK * TM * TN;
    constexpr int NLOAD = 1 + RA + RB, NSTORE = RA + RB;
    constexpr int SPM = (NLOAD + NSTORE + NMMA - 3) / (NMMA - 2);

    if (nsteps > 0) {
        load_step(0);
        store_step(0);
        if (nsteps > 1) load_step(1);
    }
    __syncthreads();
    // mode 2: loads of step + 2 and stores of step + 1; 1: stores only; 0: neither (par, mode compile-time)
    auto do_step = [&](auto par_c, auto mode_c) {
        constexpr int par = decltype(par_c)::value, mode = decltype(mode_c)::value;
        const char *As = As0 + par * BM * PITCHB, *Bs = Bs0 + par * BN * PITCHB;
        u32x4 fa[TM][NK], fb[TN][NK];
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int t = 0; t < NK; ++t)
                fa[i][t] = *reinterpret_cast<const u32x4 *>(As + a_frag + i * 32 * PITCHB + t * 32);
#pragma unroll
        for (int jn = 0; jn < TN; ++jn)
#pragma unroll
            for (int t = 0; t < NK; ++t)
                fb[jn][t] = *reinterpret_cast<const u32x4 *>(Bs + b_frag + jn * 32 * PITCHB + t * 32);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int m = 0; m < NMMA; ++m) {
            const int t = m / (TM * TN), i = (m / TN) % TM, jn = m % TN;
            acc[i][jn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fa[i][t]),
                                                                 __builtin_bit_cast(bf16x8, fb[jn][t]),
                                                                 acc[i][jn], 0, 0, 0);
            if (mode > 0 && m * SPM < NLOAD + NSTORE) {
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int q = m * SPM; q < (m + 1) * SPM && q < NLOAD + NSTORE; ++q) {
                    if (q < NLOAD) {
                        if (mode == 2) {
                            if (q == 0) slot_pos();
                            else if (q - 1 < RA) slot_a(par, q - 1);
                            else slot_b(par, q - 1 - RA);
                        }
                    } else {
                        const int w = q - NLOAD;
                        if (w < RA) store_a(par ^ 1, w);
                        else store_b(par ^ 1, w - RA);
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        if (mode > 0) __syncthreads();
    };
    using P0 = std::integral_constant<int, 0>;
    using P1 = std::integral_constant<int, 1>;
    using M2 = std::integral_constant<int, 2>;
    int step = 0;
    for (; step + 3 < nsteps; step += 2) {
        do_step(P0{}, M2{});
        do_step(P1{}, M2{});
    }
    const int rest = nsteps - step;
    if (rest == 3) {
        do_step(P0{}, M2{});
        do_step(P1{}, P1{});
        do_step(P0{}, P0{});
    } else if (rest == 2) {
        do_step(P0{}, P1{});
        do_step(P1{}, P0{});
    } else if (rest == 1) {
        do_step(P0{}, P0{});
    }

    float *out = p.part + (size_t)split * p.K * p.ncols;
#pragma unroll
    for (int jn = 0; jn < TN; ++jn) {
        const int col = n0 + (wn * TN + jn) * 32 + l32;
        if (col >= p.ncols) continue;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int row0 = m0 + (wm * TM + i) * 32 + half * 4;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = row0 + (v >> 2) * 8 + (v & 3);
                if (row < p.K) out[(size_t)row * p.ncols + col] = acc[i][jn][v];
            }
        }
    }
}

// dyp[k][e], e < row_elems: image n = e / Jy, j = e % Jy = p*Wq + q; dy(n, k, p, q) where p < P and q < Q, else 0
__global__ void pack_dy_lin(const unsigned short *__restrict__ dy, unsigned short *__restrict__ dyp, int N, int K,
                            int P, int Q, int Wq, int Jy, int row_elems, int64_t dy_bs, FastDiv div_row,
                            FastDiv div_jy, FastDiv div_wq)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (int64_t)K * row_elems) return;
    const uint32_t k = fastdiv((uint32_t)i, div_row), e = (uint32_t)i - k * (uint32_t)row_elems;
    const uint32_t n = fastdiv(e, div_jy), j = e - n * (uint32_t)Jy;
    const uint32_t pp = fastdiv(j, div_wq), q = j - pp * (uint32_t)Wq;
    unsigned short v = 0;
    if (n < (uint32_t)N && pp < (uint32_t)P && q < (uint32_t)Q) v = dy[n * dy_bs + ((int64_t)k * P + pp) * Q + q];
    dyp[i] = v;
}

// xp[c][n][e], e < Jx: padded row hh = e / Wq, column ww = e % Wq; x(n, c, hh - pad, ww - pad) where inside, else 0
__global__ void pack_x_lin(const unsigned short *__restrict__ x, unsigned short *__restrict__ xp, int N, int C, int H,
                           int W, int pad, int Wq, int Jx, int64_t x_bs, FastDiv div_jx, FastDiv div_wq)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (int64_t)C * N * Jx) return;
    const uint32_t cn = fastdiv((uint32_t)i, div_jx), e = (uint32_t)i - cn * (uint32_t)Jx;
    const uint32_t c = cn / (uint32_t)N, n = cn - c * (uint32_t)N;
    const uint32_t hh = fastdiv(e, div_wq), ww = e - hh * (uint32_t)Wq;
    const int h = (int)hh - pad, w = (int)ww - pad;
    unsigned short v = 0;
    if ((unsigned)h < (unsigned)H && (unsigned)w < (unsigned)W) v = x[n * x_bs + ((int64_t)c * H + h) * W + w];
    xp[i] = v;
}

// dw[k][c][rs] = part[0][k][rs*C + c] + part[1][k][rs*C + c] + ...  (fixed order)
// groups > 1: K filters per column; the partials of column g follow those of column g - 1, dw holds the columns'
// filters one after the other
__global__ void finish_wgrad(const float *__restrict__ part, float *__restrict__ dw, int K, int C, int RS,
                             int nsplit, int groups)
{
    const int ncols = RS * C;
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= groups * K * ncols) return;
    const int gcol = i / (K * ncols);
    i -= gcol * (K * ncols);
    part += (size_t)gcol * nsplit * K * ncols;
    dw += (size_t)gcol * K * ncols;
    const int k = i / ncols, col = i - k * ncols;
    const int rs = col / C, c = col - rs * C;
    float s = part[i];
    for (int t = 1; t < nsplit; ++t) s += part[(size_t)t * K * ncols + i];
    dw[((size_t)k * C + c) * RS + rs] = s;
}

// Sum of the split partials in a fixed order: 64 outputs per work-group; lane group g of four adds the
// splits g, g + 4, g + 8, ... in ascending order, then the four sums are added in group order.
__global__ __launch_bounds__(256) void reduce_partials(const float *__restrict__ part, float *__restrict__ dw,
                                                        int count, int nsplit)
{
    __shared__ float sums[4][64];
    const int o = threadIdx.x & 63, g = threadIdx.x >> 6;
    const int i = blockIdx.x * 64 + o;
    float s = 0.f;
    if (i < count)
        for (int k = g; k < nsplit; k += 4) s += part[(size_t)k * count + i];
    sums[g][o] = s;
    __syncthreads();
    if (g == 0 && i < count) dw[i] = ((sums[0][o] + sums[1][o]) + sums[2][o]) + sums[3][o];
}

// ---------------------------------------------------------------------------
// Fully connected layers: D[M x Nc] = sum_k A(m, k) * B(k, n) on 128 x 128 tiles
// ---------------------------------------------------------------------------
//
// x [N][I], w [O][I], y [N][O], all row-major.  The three passes as GEMMs whose
// output has its columns contiguous in memory (so a wave's stores are 128-byte
// runs):
//   forward          y [N x O]  rows n, cols o, k = i:  A = x  (k contiguous),  B = w  (k contiguous)
//   backward-data    dx[N x I]  rows n, cols i, k = o:  A = dy (k contiguous),  B = w  (cols contiguous)
//   backward-filter  dw[O x I]  rows o, cols i, k = n:  A = dy (rows contiguous), B = x (cols contiguous)
// An operand with k contiguous ("k-major") is staged in LDS as [row][16] (pitch
// 20 floats) and read with b128 like the convolution tiles.  An operand whose
// rows / columns are contiguous ("transposed") is staged as [k][128] (pitch 132
// floats: 16-byte global loads become b128 LDS writes) and each lane reads its
// eight reduction elements with ds_read_b32: lanes 0..31 take consecutive
// floats, lanes 32..63 sit 8 * 132 floats further = 32 banks further, so both
// the writes and the reads are conflict-free.  Both operands feed reduction
// element 8 * (lane / 32) + t to the t-th matrix instruction of a step.
// Register sets, LDS double buffer and load / store slots between the matrix
// instructions work as in colgemm_fast_kernel.  The reduction is cut into
// ksplit ranges (grid = tiles * ksplit); with ksplit > 1 the kernel writes
// partial sums [ksplit][M][Nc] and fc_reduce_kernel adds them in a fixed order.
struct FcArgs {
    const float *A, *B;
    float *D;              // ksplit == 1: the result (row pitch ldd); else unused
    float *part;           // ksplit > 1: partial sums [ksplit][M][Nc]
    int M, Nc, K;
    int lda, ldb, ldd;
    int mtiles, ntiles, ksplit, steps_per_split;
    const float *bias;     // forward: one value per column (output neuron), or null
    int relu;
};

template <bool AT, bool BT>
__global__ __launch_bounds__(kThreads, 2) void fc_gemm_kernel(const FcArgs p)
{
    constexpr int TM = 2, TN = 2, BM = 128, BN = 128, KC = 16;
    constexpr int PK = KC + 4;                // [row][16] pitch
    constexpr int PT = 128 + 4;               // [k][128] pitch
    constexpr int ASZ = AT ? KC * PT : BM * PK, BSZ = BT ? KC * PT : BN * PK;
    __shared__ __attribute__((aligned(16))) float As0[2 * ASZ];
    __shared__ __attribute__((aligned(16))) float Bs0[2 * BSZ];

    const int ntile = p.mtiles * p.ntiles;
    const int unit = blockIdx.x;
    const int ks = unit / ntile;
    const int tile = unit - ks * ntile;
    const int mt = tile % p.mtiles, nt = tile / p.mtiles;
    const int m0 = mt * BM, n0 = nt * BN;
    const int k_begin = ks * p.steps_per_split * KC;
    const int k_end = min(p.K, k_begin + p.steps_per_split * KC);
    const int nsteps = (k_end - k_begin + KC - 1) / KC;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = uniform(tid >> 6);
    const int wm = wave >> 1, wn = wave & 1;

    // Two 16-byte pieces per thread, operand and step.  k-major: piece q = tid + 256 * i covers row q / 4,
    // reduction elements 4 * (q % 4)..; transposed: reduction element q / 32, rows (columns) 4 * (q % 32)...
    // A piece outside the matrix or past the end of the reduction range reads the matrix base and stores zeros.
    const float *aptr[2], *bptr[2];
    int alds[2], blds[2], akoff[2], bkoff[2];
    bool arow[2], brow[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int q = tid + i * kThreads;
        if (AT) {
            const int k = q >> 5, c = (q & 31) * 4;
            arow[i] = m0 + c < p.M;
            akoff[i] = k;
            alds[i] = k * PT + c;
            aptr[i] = p.A + (size_t)(k_begin + k) * p.lda + (arow[i] ? m0 + c : 0);
        } else {
            const int row = q >> 2, kq = (q & 3) * 4;
            arow[i] = m0 + row < p.M;
            akoff[i] = kq;
            alds[i] = row * PK + kq;
            aptr[i] = p.A + (size_t)(arow[i] ? m0 + row : 0) * p.lda + k_begin + kq;
        }
        if (BT) {
            const int k = q >> 5, c = (q & 31) * 4;
            brow[i] = n0 + c < p.Nc;
            bkoff[i] = k;
            blds[i] = k * PT + c;
            bptr[i] = p.B + (size_t)(k_begin + k) * p.ldb + (brow[i] ? n0 + c : 0);
        } else {
            const int row = q >> 2, kq = (q & 3) * 4;
            brow[i] = n0 + row < p.Nc;
            bkoff[i] = kq;
            blds[i] = row * PK + kq;
            bptr[i] = p.B + (size_t)(brow[i] ? n0 + row : 0) * p.ldb + k_begin + kq;
        }
    }
    const size_t a_adv = AT ? (size_t)KC * p.lda : KC, b_adv = BT ? (size_t)KC * p.ldb : KC;

    f32x4 areg[2][2], breg[2][2];
    bool aok[2][2], bok[2][2];
    int kload = k_begin;                      // first reduction element of the next step to load
    auto slot_load = [&](int set, int q) {    // q = 0, 1: A pieces; 2, 3: B pieces (3 also advances the step)
        if (q < 2) {
            aok[set][q] = arow[q] && kload + akoff[q] < k_end;
            areg[set][q] = *reinterpret_cast<const f32x4 *>(aok[set][q] ? aptr[q] : p.A);
            aptr[q] += a_adv;
        } else {
            const int i = q - 2;
            bok[set][i] = brow[i] && kload + bkoff[i] < k_end;
            breg[set][i] = *reinterpret_cast<const f32x4 *>(bok[set][i] ? bptr[i] : p.B);
            bptr[i] += b_adv;
            if (i == 1) kload += KC;
        }
    };
    auto slot_store = [&](int set, int q) {   // the same pieces into LDS buffer `set`
        const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
        if (q < 2) *reinterpret_cast<f32x4 *>(&As0[set * ASZ + alds[q]]) = aok[set][q] ? areg[set][q] : zero;
        else *reinterpret_cast<f32x4 *>(&Bs0[set * BSZ + blds[q - 2]]) = bok[set][q - 2] ? breg[set][q - 2] : zero;
    };

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int jn = 0; jn < TN; ++jn)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][jn][v] = 0.f;

    const int l32 = lane & 31, half = lane >> 5;
    const int a_frag = AT ? half * 8 * PT + wm * 64 + l32 : (wm * 64 + l32) * PK + half * 8;
    const int b_frag = BT ? half * 8 * PT + wn * 64 + l32 : (wn * 64 + l32) * PK + half * 8;
    constexpr int NMMA = 8 * TM * TN;

    if (nsteps > 0) {
#pragma unroll
        for (int q = 0; q < 4; ++q) slot_load(0, q);
#pragma unroll
        for (int q = 0; q < 4; ++q) slot_store(0, q);
        if (nsteps > 1) {
#pragma unroll
            for (int q = 0; q < 4; ++q) slot_load(1, q);
        }
    }
    __syncthreads();

    // par / mode as in colgemm_fast_kernel: mode 2 = loads of step + 2 and stores of step + 1, 1 = stores only
    auto do_step = [&](auto par_c, auto mode_c) {
        constexpr int par = decltype(par_c)::value, mode = decltype(mode_c)::value;
        const float *As = As0 + par * ASZ, *Bs = Bs0 + par * BSZ;
        float fa[TM][8], fb[TN][8];
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            if (AT) {
#pragma unroll
                for (int t = 0; t < 8; ++t) fa[i][t] = As[a_frag + t * PT + i * 32];
            } else {
                const f32x4 *q = reinterpret_cast<const f32x4 *>(&As[a_frag + i * 32 * PK]);
                const f32x4 lo = q[0], hi = q[1];
#pragma unroll
                for (int t = 0; t < 4; ++t) { fa[i][t] = lo[t]; fa[i][4 + t] = hi[t]; }
            }
        }
#pragma unroll
        for (int jn = 0; jn < TN; ++jn) {
            if (BT) {
#pragma unroll
                for (int t = 0; t < 8; ++t) fb[jn][t] = Bs[b_frag + t * PT + jn * 32];
            } else {
                const f32x4 *q = reinterpret_cast<const f32x4 *>(&Bs[b_frag + jn * 32 * PK]);
                const f32x4 lo = q[0], hi = q[1];
#pragma unroll
                for (int t = 0; t < 4; ++t) { fb[jn][t] = lo[t]; fb[jn][4 + t] = hi[t]; }
            }
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int m = 0; m < NMMA; ++m) {
            const int t = m / (TM * TN), i = (m / TN) % TM, jn = m % TN;
            acc[i][jn] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[i][t], fb[jn][t], acc[i][jn], 0, 0, 0);
            if (mode > 0 && m < 8) {          // one slot after each of the first eight matrix instructions
                __builtin_amdgcn_sched_barrier(0);
                if (m < 4) {
                    if (mode == 2) slot_load(par, m);
                } else {
                    slot_store(par ^ 1, m - 4);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        if (mode > 0) __syncthreads();
    };
    using P0 = std::integral_constant<int, 0>;
    using P1 = std::integral_constant<int, 1>;
    using M2 = std::integral_constant<int, 2>;
    int step = 0;
    for (; step + 3 < nsteps; step += 2) {
        do_step(P0{}, M2{});
        do_step(P1{}, M2{});
    }
    const int rest = nsteps - step;
    if (rest == 3) {
        do_step(P0{}, M2{});
        do_step(P1{}, P1{});
        do_step(P0{}, P0{});
    } else if (rest == 2) {
        do_step(P0{}, P1{});
        do_step(P1{}, P0{});
    } else if (rest == 1) {
        do_step(P0{}, P0{});
    }

    // accumulator value v of block (i, jn): row 32 * i + 8 * (v / 4) + 4 * (lane / 32) + v % 4, column lane % 32
    const bool final_sums = p.ksplit == 1;
    float *out = final_sums ? p.D : p.part + (size_t)ks * p.M * p.Nc;
    const int ldo = final_sums ? p.ldd : p.Nc;
#pragma unroll
    for (int jn = 0; jn < TN; ++jn) {
        const int col = n0 + (wn * TN + jn) * 32 + l32;
        if (col >= p.Nc) continue;
        const float bv = final_sums && p.bias ? p.bias[col] : 0.f;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int row0 = m0 + (wm * TM + i) * 32 + half * 4;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = row0 + (v >> 2) * 8 + (v & 3);
                float r = acc[i][jn][v] + bv;
                if (final_sums && p.relu) r = r > 0.f ? r : 0.f;
                if (row < p.M) out[(size_t)row * ldo + col] = r;
            }
        }
    }
}

// D[m][n] = part[0][m][n] + part[1][m][n] + ... (fixed order), then bias per column and ReLU
__global__ void fc_reduce_kernel(const float *__restrict__ part, float *__restrict__ D, int nsplit, int M, int Nc,
                                 int ldd, const float *__restrict__ bias, int relu)
{
    const int64_t total = (int64_t)M * Nc;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
        float v = part[i];
        for (int k = 1; k < nsplit; ++k) v += part[(size_t)k * total + i];
        const int m = (int)(i / Nc), n = (int)(i - (int64_t)m * Nc);
        if (bias) v += bias[n];
        if (relu) v = v > 0.f ? v : 0.f;
        D[(size_t)m * ldd + n] = v;
    }
}

// SGD with momentum and weight decay, one thread per four parameters:
//   v = momentum * v - lr * (weight_decay * w + grad_scale * dw);  w += v
__global__ void sgd_update_kernel(float *__restrict__ w, const float *__restrict__ dw, float *__restrict__ vel,
                                  int64_t count, float lr, float momentum, float weight_decay, float grad_scale,
                                  int vec)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (vec) {
        const int64_t n4 = count >> 2;
        if (i < n4) {
            f32x4 wv = reinterpret_cast<f32x4 *>(w)[i];
            const f32x4 g = reinterpret_cast<const f32x4 *>(dw)[i];
            f32x4 v = reinterpret_cast<f32x4 *>(vel)[i];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                v[e] = momentum * v[e] - lr * (weight_decay * wv[e] + grad_scale * g[e]);
                wv[e] += v[e];
            }
            reinterpret_cast<f32x4 *>(vel)[i] = v;
            reinterpret_cast<f32x4 *>(w)[i] = wv;
        }
        const int64_t t = (n4 << 2) + i;      // scalar tail
        if (i < (count & 3)) {
            const float v = momentum * vel[t] - lr * (weight_decay * w[t] + grad_scale * dw[t]);
            vel[t] = v;
            w[t] += v;
        }
    } else if (i < count) {
        const float v = momentum * vel[i] - lr * (weight_decay * w[i] + grad_scale * dw[i]);
        vel[i] = v;
        w[i] += v;
    }
}

// ---------------------------------------------------------------------------
// Glue layers
// ---------------------------------------------------------------------------
// four elements per thread where the pointers allow it, scalar tail otherwise
// 16-byte groups of the element-wise kernels: 4 floats, or 8 bfloat16 widened to float
__device__ __forceinline__ void ld_vec16(const float *p, int64_t g, float (&v)[4])
{
    const f32x4 q = reinterpret_cast<const f32x4 *>(p)[g];
#pragma unroll
    for (int k = 0; k < 4; ++k) v[k] = q[k];
}
__device__ __forceinline__ void ld_vec16(const unsigned short *p, int64_t g, float (&v)[8])
{
    const u32x4 q = reinterpret_cast<const u32x4 *>(p)[g];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        v[2 * k] = __uint_as_float(q[k] << 16);
        v[2 * k + 1] = __uint_as_float(q[k] & 0xFFFF0000u);
    }
}
__device__ __forceinline__ void st_vec16(float *p, int64_t g, const float (&v)[4])
{
    reinterpret_cast<f32x4 *>(p)[g] = f32x4{v[0], v[1], v[2], v[3]};
}
__device__ __forceinline__ void st_vec16(unsigned short *p, int64_t g, const float (&v)[8])
{
    u32x4 q;
#pragma unroll
    for (int k = 0; k < 4; ++k) q[k] = (unsigned)bf16_round(v[2 * k]) | ((unsigned)bf16_round(v[2 * k + 1]) << 16);
    reinterpret_cast<u32x4 *>(p)[g] = q;
}

// One thread handles a 16-byte group (4 floats or 8 bfloat16) when `vec` (pointers 16-byte aligned), else one
// element; the last few threads of the vector form take the tail elements one each.
template <typename T>
__global__ void relu_fwd_kernel(const T *__restrict__ x, T *__restrict__ y, int64_t n, int vec)
{
    constexpr int V = 16 / (int)sizeof(T);
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (vec) {
        const int64_t nv = n / V;
        if (i < nv) {
            float v[V];
            ld_vec16(x, i, v);
#pragma unroll
            for (int k = 0; k < V; ++k) v[k] = v[k] > 0.f ? v[k] : 0.f;
            st_vec16(y, i, v);
        }
        const int64_t t = nv * V + i;
        if (i < n - nv * V) { const float v = ld_elem(x, t); st_elem(y, t, v > 0.f ? v : 0.f); }
    } else if (i < n) {
        const float v = ld_elem(x, i);
        st_elem(y, i, v > 0.f ? v : 0.f);
    }
}

template <typename T>
__global__ void relu_bwd_kernel(const T *__restrict__ x, const T *__restrict__ dy, T *__restrict__ dx, int64_t n,
                                int vec)
{
    constexpr int V = 16 / (int)sizeof(T);
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (vec) {
        const int64_t nv = n / V;
        if (i < nv) {
            float a[V], g[V];
            ld_vec16(x, i, a);
            ld_vec16(dy, i, g);
#pragma unroll
            for (int k = 0; k < V; ++k) g[k] = a[k] > 0.f ? g[k] : 0.f;
            st_vec16(dx, i, g);
        }
        const int64_t t = nv * V + i;
        if (i < n - nv * V) st_elem(dx, t, ld_elem(x, t) > 0.f ? ld_elem(dy, t) : 0.f);
    } else if (i < n) {
        st_elem(dx, i, ld_elem(x, i) > 0.f ? ld_elem(dy, i) : 0.f);
    }
}

// y[n][k][:] += b[k], in place; one thread per element (bf16 tensors: fp32 add, result rounded once)
template <typename T>
__global__ void bias_fwd_kernel(T *__restrict__ y, const float *__restrict__ b, int64_t total, int K, FastDiv div_pq,
                                FastDiv div_k)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= total) return;
    const uint32_t plane = fastdiv((uint32_t)i, div_pq);             // n * K + k
    const uint32_t k = plane - fastdiv(plane, div_k) * (uint32_t)K;
    st_elem(y, i, ld_elem(y, i) + b[k]);
}

// Bias gradient, first stage: work-group (k, s) adds dy[n][k][:] over the samples n = s, s + nsplit, ... in a
// fixed order (thread t takes positions t, t + 256, ...; then a tree over the 256 thread sums) -> part[k][s]
template <typename T>
__global__ __launch_bounds__(256) void bias_bwd_partial(const T *__restrict__ dy, float *__restrict__ part, int N,
                                                         int K, int PQ, int nsplit)
{
    __shared__ float red[256];
    const int k = blockIdx.x, sidx = blockIdx.y, tid = threadIdx.x;
    float acc = 0.f;
    for (int n = sidx; n < N; n += nsplit) {
        const T *row = dy + ((int64_t)n * K + k) * PQ;
        for (int e = tid; e < PQ; e += 256) acc += ld_elem(row, e);
    }
    red[tid] = acc;
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
        if (tid < w) red[tid] += red[tid + w];
        __syncthreads();
    }
    if (tid == 0) part[k * nsplit + sidx] = red[0];
}

// Bias gradient of one-position planes (a fully connected layer's [N][K] output gradient): thread k adds column k
// over the samples in order; neighbouring threads read neighbouring addresses.
template <typename T>
__global__ void bias_bwd_columns(const T *__restrict__ dy, float *__restrict__ db, int N, int K)
{
    const int k = blockIdx.x * blockDim.x + threadIdx.x;
    if (k >= K) return;
    float acc = 0.f;
#pragma unroll 8
    for (int n = 0; n < N; ++n) acc += ld_elem(dy, (int64_t)n * K + k);
    db[k] = acc;
}

// second stage: db[k] = part[k][0] + part[k][1] + ...
__global__ void bias_bwd_finish(const float *__restrict__ part, float *__restrict__ db, int K, int nsplit)
{
    const int k = blockIdx.x * blockDim.x + threadIdx.x;
    if (k >= K) return;
    float s = 0.f;
    for (int t = 0; t < nsplit; ++t) s += part[k * nsplit + t];
    db[k] = s;
}

// index (within the plane) of the first maximum of the 3x3 window at (2i, 2j)
template <typename T>
__device__ __forceinline__ int pool_argmax(const T *__restrict__ xp, int W, int i, int j, float &m)
{
    int best = (2 * i) * W + 2 * j;
    m = ld_elem(xp, best);
#pragma unroll
    for (int r = 0; r < 3; ++r)
#pragma unroll
        for (int s = 0; s < 3; ++s) {
            int at = (2 * i + r) * W + (2 * j + s);
            float v = ld_elem(xp, at);
            if (v > m) { m = v; best = at; }
        }
    return best;
}

template <bool RELU, typename T>
__global__ void maxpool_fwd_kernel(const T *__restrict__ x, T *__restrict__ y, int64_t total,
                                   int H, int W, int PH, int PW)
{
    int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= total) return;
    int j = (int)(t % PW);
    int64_t u = t / PW;
    int i = (int)(u % PH);
    int64_t pl = u / PH;
    float m;
    pool_argmax(x + pl * H * W, W, i, j, m);
    st_elem(y, t, RELU ? (m > 0.f ? m : 0.f) : m);
}

// Backward of the pooling (optionally of ReLU followed by pooling).  A
// work-group stages a group of whole planes in LDS and finds every window's first
// maximum once.  The gradients are then added into an LDS plane in four phases,
// one per parity class (i % 2, j % 2) of the windows: windows of one class do not
// overlap, so a phase needs no atomics, and an element always receives its (at
// most four) gradients in the same order.
// With RELU the input x is the pre-activation: the window maximum of relu(x)
// sits where the maximum of x sits whenever it is positive, and a non-positive
// maximum passes no gradient, so dx = [x > 0] * (pooled gradient routed by x).
//
// The pass is HBM-bound (read x and dy, write dx once each), so the loop is
// built to keep loads in flight: a thread holds NR elements of the next group
// of planes (and its NR/4 gradients) in registers, fetched while the current
// group is being worked on in LDS.
// group * H*W <= 256 * NR; windows are fewer than a quarter of the elements.
// A thread's unit of global access in the tiled pooling backward: one float, or two adjacent bfloat16 as
// one aligned 32-bit access.  Indices outside [0, limit) do not exist (the pair grid is shifted by
// align_shift() so that pairs are 4-byte aligned even where a plane group starts on an odd element).
__device__ __forceinline__ int align_shift(const float *) { return 0; }
__device__ __forceinline__ int align_shift(const unsigned short *p)
{
    return (int)((reinterpret_cast<uintptr_t>(p) >> 1) & 1);
}
__device__ __forceinline__ void ld_group(const float *p, int e, int limit, float (&v)[1])
{
    v[0] = e < limit ? p[e] : 0.f;
}
__device__ __forceinline__ void ld_group(const unsigned short *p, int e, int limit, float (&v)[2])
{
    if (e >= 0 && e + 1 < limit) {
        const unsigned u = *reinterpret_cast<const unsigned *>(p + e);
        v[0] = __uint_as_float(u << 16);
        v[1] = __uint_as_float(u & 0xFFFF0000u);
    } else {
        v[0] = (e >= 0 && e < limit) ? ld_elem(p, e) : 0.f;
        v[1] = (e + 1 >= 0 && e + 1 < limit) ? ld_elem(p, e + 1) : 0.f;
    }
}
__device__ __forceinline__ void st_group(float *p, int e, int limit, const float (&v)[1])
{
    if (e < limit) p[e] = v[0];
}
__device__ __forceinline__ void st_group(unsigned short *p, int e, int limit, const float (&v)[2])
{
    if (e >= 0 && e + 1 < limit) {
        *reinterpret_cast<unsigned *>(p + e) = (unsigned)bf16_round(v[0]) | ((unsigned)bf16_round(v[1]) << 16);
    } else {
        if (e >= 0 && e < limit) p[e] = bf16_round(v[0]);
        if (e + 1 >= 0 && e + 1 < limit) p[e + 1] = bf16_round(v[1]);
    }
}

template <bool RELU, int NR, typename T>
__global__ __launch_bounds__(256) void maxpool_bwd_tiled(const T *__restrict__ x, const T *__restrict__ dy,
                                                          T *__restrict__ dx, int64_t planes, int H, int W,
                                                          int PH, int PW, int group, FastDiv dPP, FastDiv dPW)
{
    constexpr int NG = NR / 4;
    constexpr int EV = 4 / (int)sizeof(T);          // adjacent elements per access: 1 float or 2 bfloat16
    static_assert(NR % EV == 0 && NG % EV == 0, "whole access groups per thread");
    // groups per thread; with pairs one more, since the pair grid may start one element early
    constexpr int KX = NR / EV + (EV > 1), KG = NG / EV + (EV > 1);
    extern __shared__ float pool_lds[];
    const int HW = H * W, PP = PH * PW;
    float *sx = pool_lds;                            // group * HW inputs
    float *sacc = pool_lds + group * HW;             // group * HW routed gradients
    const int tid = threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * group;
    float xr[KX][EV], gr[KG][EV];
    int xs = 0, gs = 0;                              // shifts of the pair grids of the fetched x and dy groups

    auto fetch = [&](int64_t pl0) {
        const int np = (int)min((int64_t)group, planes - pl0);
        const T *xg = x + pl0 * HW;
        const T *gg = dy + pl0 * PP;
        xs = align_shift(xg);
        gs = align_shift(gg);
#pragma unroll
        for (int k = 0; k < KX; ++k) ld_group(xg, EV * (tid + 256 * k) - xs, np * HW, xr[k]);
#pragma unroll
        for (int k = 0; k < KG; ++k) ld_group(gg, EV * (tid + 256 * k) - gs, np * PP, gr[k]);
    };

    int64_t pl0 = (int64_t)blockIdx.x * group;
    if (pl0 < planes) fetch(pl0);
    for (; pl0 < planes; pl0 += stride) {
        const int np = (int)min((int64_t)group, planes - pl0);
        T *og = dx + pl0 * HW;
        const int os = align_shift(og);
#pragma unroll
        for (int k = 0; k < KX; ++k)
#pragma unroll
            for (int u = 0; u < EV; ++u) {
                const int e = EV * (tid + 256 * k) - xs + u;
                if (e >= 0 && e < np * HW) { sx[e] = xr[k][u]; sacc[e] = 0.f; }
            }
        __syncthreads();
        // every window's first maximum, once; cls = parity class (i % 2, j % 2) of the window, -1 = no window
        int best[KG][EV], cls[KG][EV];
        float g[KG][EV];
#pragma unroll
        for (int k = 0; k < KG; ++k)
#pragma unroll
            for (int u = 0; u < EV; ++u) {
                const int o = EV * (tid + 256 * k) - gs + u;
                best[k][u] = 0; cls[k][u] = -1; g[k][u] = gr[k][u];
                if (o >= 0 && o < np * PP) {
                    const int pl = (int)fastdiv((uint32_t)o, dPP), rem = o - pl * PP;
                    const int i = (int)fastdiv((uint32_t)rem, dPW), j = rem - i * PW;
                    float m;
                    best[k][u] = pl * HW + pool_argmax(sx + pl * HW, W, i, j, m);
                    cls[k][u] = (i & 1) * 2 + (j & 1);
                }
            }
        if (pl0 + stride < planes) fetch(pl0 + stride);
        // windows of one parity class are disjoint (stride 2, extent 3), so within a phase every accumulator has at
        // most one writer; an element receives its up to four gradients in phase order
#pragma unroll
        for (int c = 0; c < 4; ++c) {
#pragma unroll
            for (int k = 0; k < KG; ++k)
#pragma unroll
                for (int u = 0; u < EV; ++u)
                    if (cls[k][u] == c) sacc[best[k][u]] += g[k][u];
            __syncthreads();
        }
#pragma unroll
        for (int k = 0; k < KX; ++k) {
            float res[EV];
#pragma unroll
            for (int u = 0; u < EV; ++u) {
                const int e = EV * (tid + 256 * k) - os + u;
                float sum = 0.f;
                if (e >= 0 && e < np * HW) {
                    sum = sacc[e];
                    if (RELU && !(sx[e] > 0.f)) sum = 0.f;
                }
                res[u] = sum;
            }
            st_group(og, EV * (tid + 256 * k) - os, np * HW, res);
        }
        __syncthreads();
    }
}

// Fallback for planes too large to stage: one thread per input element
// recomputes the windows that contain it.
template <bool RELU, typename T>
__global__ void maxpool_bwd_kernel(const T *__restrict__ x, const T *__restrict__ dy,
                                   T *__restrict__ dx, int64_t total, int H, int W, int PH, int PW)
{
    int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= total) return;
    int w = (int)(t % W);
    int64_t u = t / W;
    int h = (int)(u % H);
    int64_t pl = u / H;
    const T *xp = x + pl * H * W;
    const T *gp = dy + pl * PH * PW;
    const int self = h * W + w;
    int i_lo = h >= 2 ? (h - 1) / 2 : 0, i_hi = h / 2;
    int j_lo = w >= 2 ? (w - 1) / 2 : 0, j_hi = w / 2;
    if (i_hi > PH - 1) i_hi = PH - 1;
    if (j_hi > PW - 1) j_hi = PW - 1;
    float s = 0.f;
    for (int i = i_lo; i <= i_hi; ++i)
        for (int j = j_lo; j <= j_hi; ++j) {
            float m;
            if (pool_argmax(xp, W, i, j, m) == self) s += ld_elem(gp, i * PW + j);
        }
    if (RELU && !(ld_elem(xp, self) > 0.f)) s = 0.f;
    st_elem(dx, t, s);
}

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

void launch_wgrad_bf16_lin(const TileShape &t, const WgradLinArgs &a, int grid, int lds, hipStream_t st)
{
    const void *k = (t.TM == 2 && t.TN == 2) ? (const void *)wgrad_bf16_lin_kernel<2, 2, 2, 2>
                  : t.TM == 3 ? (const void *)wgrad_bf16_lin_kernel<3, 1, 1, 4>
                              : (const void *)wgrad_bf16_lin_kernel<2, 1, 1, 4>;
    if (lds > 64 * 1024) (void)hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    const dim3 g(grid), b(kThreads);
    if (t.TM == 2 && t.TN == 2) hipLaunchKernelGGL((wgrad_bf16_lin_kernel<2, 2, 2, 2>), g, b, lds, st, a);
    else if (t.TM == 3) hipLaunchKernelGGL((wgrad_bf16_lin_kernel<3, 1, 1, 4>), g, b, lds, st, a);
    else hipLaunchKernelGGL((wgrad_bf16_lin_kernel<2, 1, 1, 4>), g, b, lds, st, a);
}

void launch_wgrad_fast(const TileShape &t, const WgradFastArgs &a, const GridPlan &g, hipStream_t st)
{
    const dim3 grid(g.grid), block(kThreads);
    if (t.TM == 2 && t.TN == 2) hipLaunchKernelGGL((wgrad_fast_kernel<2, 2, 2, 2>), grid, block, g.dyn_lds, st, a);
    else if (t.TM == 3) hipLaunchKernelGGL((wgrad_fast_kernel<3, 1, 1, 4>), grid, block, g.dyn_lds, st, a);
    else if (t.TM == 2) hipLaunchKernelGGL((wgrad_fast_kernel<2, 1, 1, 4>), grid, block, g.dyn_lds, st, a);
    else hipLaunchKernelGGL((wgrad_fast_kernel<1, 2, 1, 4>), grid, block, g.dyn_lds, st, a);
}

int grid1d(int64_t n, int block) { return (int)((n + block - 1) / block); }

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
    const float *actf = fwd ? as_f32(pl.widen, act, pb.N, (int64_t)pb.C * pb.H * pb.W, &pb.x_bs, wsb, pl, 0, st)
                            : as_f32(pl.widen, act, pb.N, (int64_t)pb.K * pb.P * pb.Q, &pb.y_bs, wsb, pl, 0, st);
    const float *wf = as_f32(pl.widen_w, w, 1, w_bs, &w_bs, wsb, pl, 1, st);

    if (fast) {
        const int kc = bf ? bf16_step_channels(Cr) : pl.kc;
        const int64_t wt_elems = (int64_t)pl.Mpad * Cr * RS;
        const int GF = pl.fused_groups ? pb.groups : 1;      // columns of a grouped layer run in this one launch
        if (bf)
            hipLaunchKernelGGL(relayout_filters_cblk_bf16, dim3(grid1d(wt_elems, 256)), dim3(256), 0, st,
                               static_cast<const unsigned short *>(w), reinterpret_cast<unsigned short *>(wt), pl.M,
                               pl.Mpad, Cr / kc, RS, pb.C, fwd ? 0 : 1, kc);
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
            // channel-blocked copy of the gathered tensor: 32 bytes per position and block of 16 channels
            const int LHW = a.LH * a.LW;
            const int64_t vecs = (int64_t)pb.N * (Cr / 16) * LHW;
            u32x4 *blk = reinterpret_cast<u32x4 *>(wsb + pl.blk_off);
            hipLaunchKernelGGL(block_channels_bf16, dim3(grid1d(vecs, 256)), dim3(256), 0, st,
                               static_cast<const unsigned short *>(act), blk, pb.N, Cr, LHW, (int64_t)a.src_bs,
                               make_fastdiv((uint32_t)LHW));
            a.src = reinterpret_cast<const float *>(blk);
            a.src_bs = (Cr / 16) * LHW;
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
            hipLaunchKernelGGL(reduce_split_outputs<unsigned short>, dim3(2048), dim3(256), 0, st, a.part,
                               reinterpret_cast<unsigned short *>(a.dst), a.ksplit, per_sample, pb.N, a.dst_bs,
                               make_fastdiv((uint32_t)per_sample), a.epi_on, a.epi, a.div_plane);
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
        hipLaunchKernelGGL(pack_dy_lin, dim3(grid1d((int64_t)pb.K * row_elems, 256)), dim3(256), 0, st,
                           static_cast<const unsigned short *>(dy), dyp, pb.N, pb.K, pb.P, pb.Q, pl.lin_wq, pl.lin_jy,
                           row_elems, pb.y_bs, make_fastdiv((uint32_t)row_elems), make_fastdiv((uint32_t)pl.lin_jy),
                           make_fastdiv((uint32_t)pl.lin_wq));
        hipLaunchKernelGGL(pack_x_lin, dim3(grid1d((int64_t)pb.C * pb.N * pl.lin_jx, 256)), dim3(256), 0, st,
                           static_cast<const unsigned short *>(x), xp, pb.N, pb.C, pb.H, pb.W, pb.pad, pl.lin_wq,
                           pl.lin_jx, pb.x_bs, make_fastdiv((uint32_t)pl.lin_jx), make_fastdiv((uint32_t)pl.lin_wq));
        WgradLinArgs a;
        a.dyp = dyp; a.xp = xp; a.part = reinterpret_cast<float *>(wsb + pl.part_off);
        a.K = pb.K; a.C = pb.C; a.ncols = pl.Kg; a.S = pb.S; a.Wq = pl.lin_wq;
        a.N = pb.N; a.G = pl.lin_jy / 8; a.Jx = pl.lin_jx;
        a.row_a_bytes = row_elems * 2; a.row_x_bytes = pb.N * pl.lin_jx * 2;
        a.steps = pl.lin_steps; a.steps_per_split = pl.chunks_per_split;
        a.mtiles = pl.Mpad / pl.tile.bm();
        a.ntiles = ceil_div(pl.Kg, pl.tile.bn());
        a.nunits = a.mtiles * a.ntiles * pl.nsplit;
        const int need_lds = 2 * (pl.tile.bm() + pl.tile.bn()) * (64 * 2 + 16);
        const GridPlan g = plan_grid(a.nunits, need_lds);
        a.units_per_xcd = g.tiles_per_xcd;
        a.div_c = make_fastdiv((uint32_t)pb.C);
        a.div_s = make_fastdiv((uint32_t)pb.S);
        a.div_g = make_fastdiv((uint32_t)a.G);
        launch_wgrad_bf16_lin(pl.tile, a, g.grid, need_lds + g.dyn_lds, st);
        int rc = check_launch();
        if (rc != kStatusOk) return rc;
        const int count = pb.K * pl.Kg;
        hipLaunchKernelGGL(finish_wgrad, dim3(grid1d(count, 256)), dim3(256), 0, st, a.part, static_cast<float *>(dw),
                           pb.K, pb.C, RS, pl.nsplit, 1);
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
        const int count = pb.K * pl.Kg * GF;
        hipLaunchKernelGGL(finish_wgrad, dim3(grid1d(count, 256)), dim3(256), 0, st, a.part, static_cast<float *>(dw),
                           pb.K, pb.C, RS, pl.nsplit, GF);
        return check_launch();
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

template <bool RELU, typename T>
int pool_fwd_typed(const void *x, void *y, int64_t planes, int H, int W, int PH, int PW, hipStream_t st)
{
    const int64_t total = planes * PH * PW;
    hipLaunchKernelGGL((maxpool_fwd_kernel<RELU, T>), dim3(grid1d(total, 256)), dim3(256), 0, st,
                       static_cast<const T *>(x), static_cast<T *>(y), total, H, W, PH, PW);
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
    const int HW = H * W, PP = PH * PW;
    const T *xp = static_cast<const T *>(x), *gp = static_cast<const T *>(dy);
    T *op = static_cast<T *>(dx);
    if (HW <= 256 * 40) {
        // planes staged whole: up to 16 elements per thread (several small planes), else one plane of up to 40
        const bool small = HW <= 256 * 16;
        const int group = small ? (256 * 16) / HW : 1;
        int64_t blocks = (planes + group - 1) / group;
        if (blocks > 256 * 6) blocks = 256 * 6;
        const size_t lds = (size_t)group * HW * 8;        // inputs + accumulators
        const FastDiv dPP = make_fastdiv(PP), dPW = make_fastdiv(PW);
        if (small) {
            hipLaunchKernelGGL((maxpool_bwd_tiled<RELU, 16, T>), dim3((int)blocks), dim3(256), lds, st, xp, gp, op,
                               planes, H, W, PH, PW, group, dPP, dPW);
        } else {
            if (lds > 64 * 1024)
                (void)hipFuncSetAttribute(reinterpret_cast<const void *>(maxpool_bwd_tiled<RELU, 40, T>),
                                          hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
            hipLaunchKernelGGL((maxpool_bwd_tiled<RELU, 40, T>), dim3((int)blocks), dim3(256), lds, st, xp, gp, op,
                               planes, H, W, PH, PW, group, dPP, dPW);
        }
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

#ifdef CONVNET_PHASE_PROBE
extern "C" int conv_debug_set_probe(void *buf)
{
    long long *p = static_cast<long long *>(buf);
    return (int)hipMemcpyToSymbol(HIP_SYMBOL(g_probe), &p, sizeof(p));
}
#endif

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
    for (int g = 0; g < groups; ++g) {
        const char *pa = static_cast<const char *>(a), *pbp = static_cast<const char *>(b);
        char *po = static_cast<char *>(out);
        if (op == kOpFwd) { pa += g * pb.x_gs * in_b; pbp += g * pb.w_gs * in_b; po += g * pb.y_gs * out_b; }
        else if (op == kOpBwdData) { pa += g * pb.y_gs * in_b; pbp += g * pb.w_gs * in_b; po += g * pb.x_gs * out_b; }
        else { pa += g * pb.x_gs * in_b; pbp += g * pb.y_gs * in_b; po += g * pb.w_gs * 4; }
        // column bases must keep the alignment the kernels rely on
        if (!aligned(pa, 16) || !aligned(pbp, 16) || !aligned(po, 16)) return kErrMisaligned;
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

}  // extern "C"
