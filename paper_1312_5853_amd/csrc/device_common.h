// Tap table, filter re-layouts, element conversions, the epilogue, and the shared MFMA step.
// Part of convnet_hotpath.hip: included there, inside its anonymous namespace, after the common
// definitions (kThreads, kPitch, vector types); not a stand-alone header.
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
