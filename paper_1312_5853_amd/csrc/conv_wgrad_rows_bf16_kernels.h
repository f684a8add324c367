// Backward-filter for a stride-4 layer with few input channels (the 11x11 first layer) and bf16 tensors, on the
// bf16 matrix instruction.  Part of convnet_hotpath.hip: included there, inside its anonymous namespace, after
// conv_bf16_dma_kernels.h.
//
// GEMM view: dw[k][(c, r, s)] = sum over (n, p, q) of dy[n][k][p][q] * x[n][c][4p + r - 2][4q + s - 2], fp32 sums.
// v_mfma_f32_32x32x16_bf16 wants, per lane, eight CONSECUTIVE reduction indices of one row (one column) in a
// register quad.  The reduction runs along q inside one output row p (at most 64 positions, processed as
// 16-position blocks, zero beyond Q).  dy is contiguous along q; x is not (stride 4).  So every input row is
// staged in LDS once as S de-interleaved, shifted copies
//     E[c][row][s][q] = x[c][row - 2][4q + s - 2]            (zero outside the image, q = 0..63)
// and the operand of tap (c, r, s) for output row p is E[c][4p + r][s][q0 .. q0 + 7]: sixteen aligned bytes.  An
// input row is built once and serves every (p, r) pair that reads it: the rows live in a ring of 16 per channel,
// and a step (one output row p) adds the four rows the next step needs while the matrix instructions run.
// Building a row costs ~4 v_perm_b32 and one 16-byte LDS store per 8 outputs; the rows of dy (arbitrary 2-byte
// alignment in memory) are read as 4-byte-aligned words and shifted into place with v_alignbit_b32.
//
// One work-group (four waves) per CU owns the whole 96 x 384 result for its share of (image, output-row range)
// units: 3 x 3 blocks of 32 x 32 per wave, 144 accumulator registers, no reduction over work-groups inside the
// kernel.  Each work-group writes one partial result; reduce_partials adds them in a fixed order.
// LDS rows are 144 bytes (64 positions + 16): the 16 lanes of a ds_read_b128 phase read 16 consecutive filters
// (pitch 144) or 16 consecutive taps (pitch 144 per s, S * 144 per r), which covers the 64 banks once for S = 11.
constexpr int kRowsPitch = 144;            // bytes of 64 positions in LDS plus padding
constexpr int kRowsM = 96;                 // filters per work-group (three 32-row blocks)
constexpr int kRowsRing = 16;              // staged input rows per channel
constexpr int kRowsCols = 384;             // taps per work-group (four waves x three 32-column blocks)
constexpr int kRowsABuf = kRowsM * kRowsPitch;

struct WgradRowsArgs {
    const unsigned short *x, *dy;
    float *part;                 // [work-group][K][Kg]
    int N, C, H, W, K, R, S, P, Q, Kg;         // stride 4, pad 2
    int64_t x_bs, y_bs;          // elements between images
    int64_t dy_elems;            // elements of dy that may be read: (N - 1) * y_bs + K * P * Q
    int splits, units;           // output-row ranges per image; units = N * splits
    int ng;                      // groups of 8 positions per output row: ceil(Q / 8)
    int nkb;                     // 16-position blocks per output row: ceil(Q / 16)
    int nnew;                    // input rows a step adds per channel: min(R, 4)
    FastDiv div_splits, div_ng;
};

typedef unsigned int u32x4_a4 __attribute__((ext_vector_type(4), aligned(4)));

// mask of output word i (elements 2i, 2i + 1) of a group of eight of which the first nv are real
__device__ __forceinline__ unsigned rows_mask(int nv, int i)
{
    return (2 * i < nv ? 0x0000FFFFu : 0u) | (2 * i + 1 < nv ? 0xFFFF0000u : 0u);
}

// The copies s = 6*HF .. 6*HF + 5 (s < S) of eight positions, from the window of five 16-byte pieces that starts
// at input column 32g - 8 + 8*HF: position i of copy s is window element 4i + s + 6 - 8*HF.
template <int HF>
__device__ __forceinline__ void rows_store_copies(const u32x4 (&win)[5], char *dst, int S, int nv)
{
    unsigned w[20];
#pragma unroll
    for (int k = 0; k < 5; ++k)
#pragma unroll
        for (int i = 0; i < 4; ++i) w[4 * k + i] = win[k][i];
    unsigned mask[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) mask[i] = rows_mask(nv, i);
#pragma unroll
    for (int sl = 0; sl < 6 - HF; ++sl) {
        const int s = 6 * HF + sl;
        const int o = ((s + 6) >> 1) - 4 * HF;                     // word of element 0 of this copy
        const unsigned sel = (s & 1) ? 0x07060302u : 0x05040100u;  // high or low halves of the two words
        if (s < S) {
            u32x4 out;
#pragma unroll
            for (int j = 0; j < 4; ++j) out[j] = __builtin_amdgcn_perm(w[4 * j + 2 + o], w[4 * j + o], sel) & mask[j];
            *reinterpret_cast<u32x4 *>(dst + s * kRowsPitch) = out;
        }
    }
}

__global__ __launch_bounds__(256, 1) void wgrad_rows_bf16_kernel(const WgradRowsArgs p)
{
    extern __shared__ __attribute__((aligned(16))) float lds_fast[];
    char *const lds = reinterpret_cast<char *>(lds_fast);      // dy rows, buffer 0 | buffer 1 | E
    char *const E = lds + 2 * kRowsABuf;
    const int tid = threadIdx.x, lane = tid & 63, wave = uniform(tid >> 6);
    const int l32 = lane & 31, half = lane >> 5;
    const int erow = p.S * kRowsPitch;                         // one staged input row: S copies
    const int echan = kRowsRing * erow;
    const int lds_bytes = 2 * kRowsABuf + p.C * echan;

    // positions >= 8 * ng are never written again: zero once
    for (int o = tid * 16; o < lds_bytes; o += 256 * 16) *reinterpret_cast<u32x4 *>(lds + o) = u32x4{0u, 0u, 0u, 0u};

    // this lane's three taps: byte offset of (c, ring row 0, s) in E and the filter row r
    int tap_off[3], tap_r[3];
#pragma unroll
    for (int t = 0; t < 3; ++t) {
        const int j = 32 * (3 * wave + t) + l32;
        const int jj = j < p.Kg ? j : 0;                       // columns beyond the filter read tap 0, never stored
        const int c = jj / (p.R * p.S), rs = jj - c * (p.R * p.S);
        const int r = rs / p.S, s = rs - r * p.S;
        tap_off[t] = c * echan + s * kRowsPitch + half * 16;
        tap_r[t] = r;
    }

    // E building: waves 0, 2 make the copies s = 0..5 and waves 1, 3 the copies s = 6..10 of one (row, group of 8
    // positions) pair per lane
    const int hf = wave & 1;
    const int pair = (wave >> 1) * 64 + lane;
    // Loads and their use are kept apart (the loads of the next step are in flight while this step's matrix
    // instructions run): a load always reads a valid address, and what lies outside the image becomes zero only
    // when the piece is consumed.  Returns the mask of pieces that are inside.
    auto e_load = [&](u32x4 (&win)[5], int n, int c, int hh, int g, bool on) -> unsigned {
        const int h = hh - 2;
        const bool rok = on & ((unsigned)h < (unsigned)p.H);
        const unsigned short *row = p.x + (size_t)n * p.x_bs + ((size_t)c * p.H + (rok ? h : 0)) * p.W;
        unsigned inside = 0;
#pragma unroll
        for (int k = 0; k < 5; ++k) {
            const int start = 32 * g - 8 + 8 * (hf + k);        // W is a multiple of 8: a piece is inside or outside
            const bool ok = rok & ((unsigned)start < (unsigned)p.W);
            win[k] = *reinterpret_cast<const u32x4 *>(row + (ok ? start : 0));
            inside |= ok ? 1u << k : 0u;
        }
        return inside;
    };
    auto e_store = [&](u32x4 (&win)[5], unsigned inside, int c, int hh, int g) {
#pragma unroll
        for (int k = 0; k < 5; ++k)
            if (!(inside >> k & 1)) win[k] = u32x4{0u, 0u, 0u, 0u};
        char *dst = E + c * echan + (hh & (kRowsRing - 1)) * erow + g * 16;
        const int nv = min(max(p.Q - 8 * g, 0), 8);
        if (hf) rows_store_copies<1>(win, dst, p.S, nv);
        else rows_store_copies<0>(win, dst, p.S, nv);
    };
    // steady state: the nnew rows a step adds, per channel (c, i) and group g: fixed per lane
    const int npairs_new = p.C * p.nnew * p.ng;
    const bool e_on = pair < npairs_new;
    int e_c, e_i, e_g;
    {
        const int pp = e_on ? pair : 0;
        const int t = (int)fastdiv((uint32_t)pp, p.div_ng);
        e_g = pp - t * p.ng;
        e_c = t / p.nnew;
        e_i = t - e_c * p.nnew;
    }

    // dy rows: item (filter m, group j of 8 positions), three per thread; rows beyond K repeat row K - 1 (their
    // sums are never stored)
    const int nitems = kRowsM * p.ng;
    int a_base[3], a_dst[3], a_nv[3];
#pragma unroll
    for (int u = 0; u < 3; ++u) {
        const int it = min(tid + 256 * u, nitems - 1);
        const int m = (int)fastdiv((uint32_t)it, p.div_ng), j = it - m * p.ng;
        a_base[u] = min(m, p.K - 1) * p.P * p.Q + 8 * j;
        a_dst[u] = m * kRowsPitch + j * 16;
        a_nv[u] = min(max(p.Q - 8 * j, 0), 8);
    }
    // Five 4-byte words from the even element at or below the item's first one.  Where those 20 bytes would pass
    // the end of the tensor (the last group of its last row) the load reads element 0 instead and the item is
    // fetched one element at a time when it is consumed (tail[u] = its first even element, else -1).
    auto a_load = [&](unsigned (&d)[3][5], int (&sh)[3], int64_t (&tail)[3], int n, int prow) {
        const int64_t rowbase = (int64_t)n * p.y_bs + (int64_t)prow * p.Q;
#pragma unroll
        for (int u = 0; u < 3; ++u) {
            const int64_t o = rowbase + a_base[u];
            const int64_t oe = o & ~(int64_t)1;                 // 4-byte aligned element
            sh[u] = (int)(o & 1) * 16;
            const bool fits = oe + 10 <= p.dy_elems;
            tail[u] = fits ? -1 : oe;
            const unsigned short *src = p.dy + (fits ? oe : 0);
            const u32x4_a4 v = *reinterpret_cast<const u32x4_a4 *>(src);
            d[u][0] = v[0]; d[u][1] = v[1]; d[u][2] = v[2]; d[u][3] = v[3];
            d[u][4] = *reinterpret_cast<const unsigned *>(src + 8);
        }
    };
    auto a_store = [&](unsigned (&d)[3][5], const int (&sh)[3], const int64_t (&tail)[3], int buf) {
#pragma unroll
        for (int u = 0; u < 3; ++u) {
            if (tid + 256 * u < nitems) {
                if (tail[u] >= 0) {
#pragma unroll
                    for (int i = 0; i < 5; ++i) {
                        const int64_t e = tail[u] + 2 * i;
                        const unsigned lo = e < p.dy_elems ? p.dy[e] : 0u;
                        const unsigned hi = e + 1 < p.dy_elems ? p.dy[e + 1] : 0u;
                        d[u][i] = lo | (hi << 16);
                    }
                }
                u32x4 out;
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    out[i] = __builtin_amdgcn_alignbit(d[u][i + 1], d[u][i], (unsigned)sh[u]) & rows_mask(a_nv[u], i);
                *reinterpret_cast<u32x4 *>(lds + buf * kRowsABuf + a_dst[u]) = out;
            }
        }
    };

    f32x16 acc[3][3];
#pragma unroll
    for (int i = 0; i < 3; ++i)
#pragma unroll
        for (int t = 0; t < 3; ++t)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][t][v] = 0.f;

    auto compute = [&](int prow, int buf) {
        const char *Ab = lds + buf * kRowsABuf + l32 * kRowsPitch + half * 16;
        const char *Bb[3];
#pragma unroll
        for (int t = 0; t < 3; ++t) Bb[t] = E + tap_off[t] + ((4 * prow + tap_r[t]) & (kRowsRing - 1)) * erow;
        bf16x8 fa[2][3], fb[2][3];
        auto read = [&](int set, int kb) {
#pragma unroll
            for (int i = 0; i < 3; ++i)
                fa[set][i] = *reinterpret_cast<const bf16x8 *>(Ab + i * 32 * kRowsPitch + kb * 32);
#pragma unroll
            for (int t = 0; t < 3; ++t) fb[set][t] = *reinterpret_cast<const bf16x8 *>(Bb[t] + kb * 32);
        };
        read(0, 0);
#pragma unroll
        for (int kb = 0; kb < 4; ++kb) {
            if (kb < p.nkb) {
                if (kb + 1 < p.nkb) read((kb + 1) & 1, kb + 1);
#pragma unroll
                for (int i = 0; i < 3; ++i)
#pragma unroll
                    for (int t = 0; t < 3; ++t)
                        acc[i][t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[kb & 1][i], fb[kb & 1][t], acc[i][t],
                                                                            0, 0, 0);
            }
        }
    };

    for (int unit = blockIdx.x; unit < p.units; unit += gridDim.x) {
        const int n = (int)fastdiv((uint32_t)unit, p.div_splits);
        const int sp = unit - n * p.splits;
        const int p_begin = (int)((int64_t)p.P * sp / p.splits), p_end = (int)((int64_t)p.P * (sp + 1) / p.splits);
        if (p_begin >= p_end) continue;
        __syncthreads();                                        // zero fill / the previous unit's reads are done
        // every input row of the first output row, and its dy rows
        {
            const int total = p.C * p.R * p.ng;
            for (int q0 = 0; q0 < total; q0 += 128) {
                const int pi = q0 + pair;
                const bool on = pi < total;
                const int pp = on ? pi : 0;
                const int t = (int)fastdiv((uint32_t)pp, p.div_ng);
                const int g = pp - t * p.ng, c = t / p.R, i = t - c * p.R;
                u32x4 win[5];
                const unsigned inside = e_load(win, n, c, 4 * p_begin + i, g, on);
                if (on) e_store(win, inside, c, 4 * p_begin + i, g);
            }
            unsigned d[3][5];
            int sh[3];
            int64_t tail[3];
            a_load(d, sh, tail, n, p_begin);
            a_store(d, sh, tail, 0);
        }
        __syncthreads();
        int buf = 0;
        for (int prow = p_begin; prow < p_end; ++prow) {
            const bool more = prow + 1 < p_end;
            // rows of the next step: loads now, LDS stores after this step's matrix instructions
            const int hh_new = 4 * (prow + 1) + p.R - p.nnew + e_i;
            u32x4 win[5];
            unsigned d[3][5], inside = 0;
            int sh[3];
            int64_t tail[3];
            if (more) {
                inside = e_load(win, n, e_c, hh_new, e_g, e_on);
                a_load(d, sh, tail, n, prow + 1);
            }
            compute(prow, buf);
            if (more) {
                if (e_on) e_store(win, inside, e_c, hh_new, e_g);
                a_store(d, sh, tail, buf ^ 1);
            }
            __syncthreads();
            buf ^= 1;
        }
    }

    float *out = p.part + (size_t)blockIdx.x * p.K * p.Kg;
#pragma unroll
    for (int i = 0; i < 3; ++i)
#pragma unroll
        for (int t = 0; t < 3; ++t) {
            const int col = 32 * (3 * wave + t) + l32;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = 32 * i + (v >> 2) * 8 + half * 4 + (v & 3);
                if (row < p.K && col < p.Kg) out[(size_t)row * p.Kg + col] = acc[i][t][v];
            }
        }
}
