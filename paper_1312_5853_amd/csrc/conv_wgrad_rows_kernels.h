// Backward-filter for layers with few input channels (the 11x11 stride-4 first layer): a work-group keeps the whole
// K x (C*R*S) result in registers and walks the output rows of its share of the images with the input rows staged in
// LDS.  Two kernels: bf16 tensors on the bf16 matrix instruction (stride 4, pad 2; below) and fp32 tensors on the
// fp32 matrix instruction (second half of the file).
// Part of convnet_hotpath.hip: included there, inside its anonymous namespace, after conv_bf16_dma_kernels.h.
//
// --- bf16 ---
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
// LDS bytes behind E that idle lanes store to (lane L at L * 16 + s * kRowsPitch, s <= 10): the steady-state step has
// no branch around a store, so that matrix instructions, the staging arithmetic and the LDS stores can be interleaved
constexpr int kRowsTrash = 255 * 16 + 10 * kRowsPitch + 16;

struct WgradRowsArgs {
    const unsigned short *x, *dy;
    float *part;                 // [work-group][K][Kg]
    int N, C, H, W, K, R, S, P, Q, Kg;         // stride 4, pad 2
    int x_bs, y_bs;              // elements between images (every offset into x and dy fits 31 bits)
    int dy_elems;                // elements of dy that may be read: (N - 1) * y_bs + K * P * Q
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

// Copy s of eight positions from the window of six 16-byte pieces that starts at input column 32g - 8:
// position i of copy s is window element 4i + s + 6.
template <int S_>
__device__ __forceinline__ void rows_store_copy(const u32x4 (&win)[6], char *dst, const unsigned (&mask)[4])
{
    constexpr int o = (S_ + 6) >> 1;                                // word of element 0 of this copy
    constexpr unsigned sel = (S_ & 1) ? 0x07060302u : 0x05040100u;  // high or low halves of the two words
    u32x4 out;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const unsigned lo = win[(4 * j + o) >> 2][(4 * j + o) & 3], hi = win[(4 * j + 2 + o) >> 2][(4 * j + 2 + o) & 3];
        out[j] = __builtin_amdgcn_perm(hi, lo, sel) & mask[j];
    }
    *reinterpret_cast<u32x4 *>(dst + S_ * kRowsPitch) = out;
}

// FULL: S = 11 and Q in 49..64 (four 16-position blocks), the first layer's case: those two are compile-time, and
// the LDS stores of the next row sit between the matrix instructions.
template <bool FULL>
__global__ __launch_bounds__(256, 1) void wgrad_rows_bf16_kernel(const WgradRowsArgs p)
{
    extern __shared__ __attribute__((aligned(16))) float lds_fast[];
    char *const lds = reinterpret_cast<char *>(lds_fast);      // dy rows, buffer 0 | buffer 1 | E
    char *const E = lds + 2 * kRowsABuf;
    const int tid = threadIdx.x, lane = tid & 63, wave = uniform(tid >> 6);
    const int l32 = lane & 31, half = lane >> 5;
    const int S = FULL ? 11 : p.S, nkb = FULL ? 4 : p.nkb;
    const int erow = S * kRowsPitch;                           // one staged input row: S copies
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
        const int c = jj / (p.R * S), rs = jj - c * (p.R * S);
        const int r = rs / S, s = rs - r * S;
        tap_off[t] = c * echan + s * kRowsPitch + half * 16;
        tap_r[t] = r;
    }

    // E building: one (input row, group of 8 positions) pair per lane: six 16-byte pieces of the
    // row in (the window: input columns 32g - 8 .. 32g + 39), S copies out.  Loads and their use are kept apart (a
    // row is loaded three steps before it is needed): a load always reads a valid address -- a piece outside the row
    // reads the row's first piece, a row outside the image reads row 0 -- and zeros are put in when the window is
    // consumed.  Only two words of a window can hold padding that a real position reads: word 3 (columns -2, -1, for
    // g = 0) and word 0 of the piece that starts at column W (columns W, W + 1); everything else outside the row
    // only feeds positions >= Q, which the position masks clear.  FULL uses that; the general variant clears whole
    // pieces.
    auto e_load = [&](u32x4 (&win)[6], const char *img, int c, int hh, int g, bool on) {
        const int h = hh - 2;
        const bool rok = on & ((unsigned)h < (unsigned)p.H);
        const unsigned rowb = (unsigned)((c * p.H + (rok ? h : 0)) * p.W) * 2u;
#pragma unroll
        for (int k = 0; k < 6; ++k) {
            const int start = 32 * g - 8 + 8 * k;               // W is a multiple of 8: a piece is inside or outside
            const bool ok = (unsigned)start < (unsigned)p.W;
            win[k] = *reinterpret_cast<const u32x4 *>(img + (size_t)(rowb + (ok ? (unsigned)start * 2u : 0u)));
        }
    };
    // zeros for what lies outside the image; the position masks of the group
    auto e_prepare = [&](u32x4 (&win)[6], unsigned (&mask)[4], int hh, int g) {
        const bool rok = (unsigned)(hh - 2) < (unsigned)p.H;
        if (FULL) {
            if (g == 0) win[0][3] = 0u;
#pragma unroll
            for (int k = 1; k < 6; ++k)
                if (32 * g - 8 + 8 * k == p.W) win[k][0] = 0u;
        } else {
#pragma unroll
            for (int k = 0; k < 6; ++k)
                if (!((unsigned)(32 * g - 8 + 8 * k) < (unsigned)p.W)) win[k] = u32x4{0u, 0u, 0u, 0u};
        }
        const int nv = rok ? min(max(p.Q - 8 * g, 0), 8) : 0;  // a row outside the image: every position zero
#pragma unroll
        for (int i = 0; i < 4; ++i) mask[i] = rows_mask(nv, i);
    };
    auto e_dst = [&](int c, int hh, int g) { return E + c * echan + (hh & (kRowsRing - 1)) * erow + g * 16; };
    char *const trash = E + p.C * echan + tid * 16;
    auto e_copy = [&](auto s_c, const u32x4 (&win)[6], char *dst, const unsigned (&mask)[4]) {
        constexpr int S_ = decltype(s_c)::value;
        if (S_ < S) rows_store_copy<S_>(win, dst, mask);
    };
    auto e_store_all = [&](u32x4 (&win)[6], int c, int hh, int g) {
        unsigned mask[4];
        e_prepare(win, mask, hh, g);
        char *dst = e_dst(c, hh, g);
        e_copy(std::integral_constant<int, 0>{}, win, dst, mask); e_copy(std::integral_constant<int, 1>{}, win, dst, mask);
        e_copy(std::integral_constant<int, 2>{}, win, dst, mask); e_copy(std::integral_constant<int, 3>{}, win, dst, mask);
        e_copy(std::integral_constant<int, 4>{}, win, dst, mask); e_copy(std::integral_constant<int, 5>{}, win, dst, mask);
        e_copy(std::integral_constant<int, 6>{}, win, dst, mask); e_copy(std::integral_constant<int, 7>{}, win, dst, mask);
        e_copy(std::integral_constant<int, 8>{}, win, dst, mask); e_copy(std::integral_constant<int, 9>{}, win, dst, mask);
        e_copy(std::integral_constant<int, 10>{}, win, dst, mask);
    };
    // steady state: the nnew rows a step adds, per channel (c, i) and group g: fixed per lane
    // (eight lanes per row, lane g of them idle for g >= ng: the 16-byte LDS stores of eight consecutive lanes then
    // go to one row's 128 consecutive bytes and never meet a bank twice)
    const int e_g = tid & 7;
    const bool e_on = (tid >> 3) < p.C * p.nnew && e_g < p.ng;
    int e_c, e_i;
    {
        const int t = e_on ? tid >> 3 : 0;
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
    // fetched one element at a time when it is consumed.
    unsigned a_mask[3][4];
#pragma unroll
    for (int u = 0; u < 3; ++u)
#pragma unroll
        for (int i = 0; i < 4; ++i) a_mask[u][i] = rows_mask(a_nv[u], i);
    const char *const dyb = reinterpret_cast<const char *>(p.dy);
    auto a_load = [&](unsigned (&d)[3][5], int n, int prow) {
        const int rowbase = n * p.y_bs + prow * p.Q;
#pragma unroll
        for (int u = 0; u < 3; ++u) {
            const int oe = (rowbase + a_base[u]) & ~1;          // 4-byte aligned element
            const unsigned off = oe + 10 <= p.dy_elems ? (unsigned)oe * 2u : 0u;
            const u32x4_a4 v = *reinterpret_cast<const u32x4_a4 *>(dyb + (size_t)off);
            d[u][0] = v[0]; d[u][1] = v[1]; d[u][2] = v[2]; d[u][3] = v[3];
            d[u][4] = *reinterpret_cast<const unsigned *>(dyb + (size_t)off + 16);
        }
    };
    auto a_shift_store = [&](int u, const unsigned (&d)[5], int o, char *dst) {
        const unsigned sh = (unsigned)(o & 1) * 16;
        u32x4 out;
#pragma unroll
        for (int i = 0; i < 4; ++i) out[i] = __builtin_amdgcn_alignbit(d[i + 1], d[i], sh) & a_mask[u][i];
        *reinterpret_cast<u32x4 *>(dst) = out;
    };
    // no branch: a thread without an item u stores to the trash area; an item at the tensor's end stores what the
    // clamped load returned and is put right by a_fix_tail before the barrier
    auto a_store_fast = [&](int u, const unsigned (&d)[5], int n, int prow, int buf) {
        char *dst = tid + 256 * u < nitems ? lds + buf * kRowsABuf + a_dst[u] : trash;
        a_shift_store(u, d, n * p.y_bs + prow * p.Q + a_base[u], dst);
    };
    auto a_fix_tail = [&](int n, int prow, int buf) {
#pragma unroll
        for (int u = 0; u < 3; ++u) {
            const int o = n * p.y_bs + prow * p.Q + a_base[u];
            const int oe = o & ~1;
            if (tid + 256 * u < nitems && oe + 10 > p.dy_elems) {   // elements past the end lie beyond Q: masked
                unsigned d[5];
#pragma unroll
                for (int i = 0; i < 5; ++i) {
                    const unsigned lo = p.dy[min(oe + 2 * i, p.dy_elems - 1)];
                    const unsigned hi = p.dy[min(oe + 2 * i + 1, p.dy_elems - 1)];
                    d[i] = lo | (hi << 16);
                }
                a_shift_store(u, d, o, lds + buf * kRowsABuf + a_dst[u]);
            }
        }
    };
    // rows whose items can reach the tensor's end (a superset; a_fix_tail tests each item)
    auto near_end = [&](int n, int prow) { return n == p.N - 1 && (p.P - prow) * p.Q <= 8 * p.ng + 12; };
    auto a_store_one = [&](int u, const unsigned (&d)[5], int n, int prow, int buf) {
        if (tid + 256 * u < nitems) a_store_fast(u, d, n, prow, buf);
    };

    f32x16 acc[3][3];
#pragma unroll
    for (int i = 0; i < 3; ++i)
#pragma unroll
        for (int t = 0; t < 3; ++t)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][t][v] = 0.f;

    // three register stages: stage (row - p_begin) % 3 holds the loads of that output row
    u32x4 win[3][6];
    unsigned dd[3][3][5];

    for (int unit = blockIdx.x; unit < p.units; unit += gridDim.x) {
        const int n = (int)fastdiv((uint32_t)unit, p.div_splits);
        const int sp = unit - n * p.splits;
        const int p_begin = (int)((int64_t)p.P * sp / p.splits), p_end = (int)((int64_t)p.P * (sp + 1) / p.splits);
        if (p_begin >= p_end) continue;
        __syncthreads();                                        // zero fill / the previous unit's reads are done
        const char *const img = reinterpret_cast<const char *>(p.x + (size_t)n * p.x_bs);
        auto issue = [&](auto st_c, int prow) {                 // loads of output row prow (clamped to the unit)
            constexpr int ST = decltype(st_c)::value;
            const int pr = min(prow, p_end - 1);
            e_load(win[ST], img, e_c, 4 * pr + p.R - p.nnew + e_i, e_g, e_on);
            a_load(dd[ST], n, pr);
        };
        // every input row of the first output row, and its dy rows
        {
            const int rows = p.C * p.R;
            for (int t0 = 0; t0 < rows; t0 += 32) {
                const int t1 = t0 + (tid >> 3), g = tid & 7;
                const bool on = t1 < rows && g < p.ng;
                const int t = on ? t1 : 0;
                const int c = t / p.R, i = t - c * p.R;
                e_load(win[0], img, c, 4 * p_begin + i, g, on);
                if (on) e_store_all(win[0], c, 4 * p_begin + i, g);
            }
            a_load(dd[0], n, p_begin);
#pragma unroll
            for (int u = 0; u < 3; ++u) a_store_one(u, dd[0][u], n, p_begin, 0);
            if (near_end(n, p_begin)) a_fix_tail(n, p_begin, 0);
        }
        issue(std::integral_constant<int, 1>{}, p_begin + 1);
        issue(std::integral_constant<int, 2>{}, p_begin + 2);
        __syncthreads();
        int buf = 0;
        // One output row: loads of row prow + 3 into the stage row prow used; matrix instructions of row prow; the
        // stage of row prow + 1 goes to LDS (dy buffer buf ^ 1, ring rows no tap of row prow reads).  After the last
        // row of the unit the stores repeat that row into places nothing reads before they are rewritten.
        auto step = [&](auto st_c, int prow) {
            constexpr int ST = decltype(st_c)::value, SN = (ST + 1) % 3;
            issue(st_c, prow + 3);
            const int pn = min(prow + 1, p_end - 1);            // the row stage SN holds
            const int hh_new = 4 * (prow + 1) + p.R - p.nnew + e_i;
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
            unsigned mask[4];
            char *dst = e_on ? e_dst(e_c, hh_new, e_g) : trash;
            // store work in twelve slots: copy s of the new input rows in slot s, a dy item in slots 3, 7, 11.
            // FULL: no branches (idle lanes store to the trash area), so the whole step is one scheduling region
            auto slot = [&](auto k_c) {
                constexpr int K_ = decltype(k_c)::value;
                // (the four words of the window no copy reads stay allocated until here: the register allocator would
                // otherwise hand them out while their load is in flight, and every such reuse waits for the load)
                if (K_ == 0)
                    asm volatile("" :: "v"(win[SN][0][0]), "v"(win[SN][0][1]), "v"(win[SN][0][2]), "v"(win[SN][5][3]));
                if (FULL) {
                    if (K_ == 0) e_prepare(win[SN], mask, 4 * pn + p.R - p.nnew + e_i, e_g);
                    if (K_ < 11) e_copy(std::integral_constant<int, K_ < 11 ? K_ : 0>{}, win[SN], dst, mask);
                    if (K_ % 4 == 3) a_store_fast(K_ / 4, dd[SN][K_ / 4], n, pn, buf ^ 1);
                } else {
                    if (K_ == 0 && e_on) e_prepare(win[SN], mask, 4 * pn + p.R - p.nnew + e_i, e_g);
                    if (K_ < 11 && e_on) e_copy(std::integral_constant<int, K_ < 11 ? K_ : 0>{}, win[SN], dst, mask);
                    if (K_ % 4 == 3) a_store_one(K_ / 4, dd[SN][K_ / 4], n, pn, buf ^ 1);
                }
            };
            read(0, 0);
            if (FULL) {
#pragma unroll
                for (int kb = 0; kb < 4; ++kb) {
                    if (kb + 1 < 4) read((kb + 1) & 1, kb + 1);
#pragma unroll
                    for (int i = 0; i < 3; ++i) {
#pragma unroll
                        for (int t = 0; t < 3; ++t)
                            acc[i][t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[kb & 1][i], fb[kb & 1][t], acc[i][t],
                                                                                0, 0, 0);
                        if (kb == 0) { if (i == 0) slot(std::integral_constant<int, 0>{}); if (i == 1) slot(std::integral_constant<int, 1>{}); if (i == 2) slot(std::integral_constant<int, 2>{}); }
                        if (kb == 1) { if (i == 0) slot(std::integral_constant<int, 3>{}); if (i == 1) slot(std::integral_constant<int, 4>{}); if (i == 2) slot(std::integral_constant<int, 5>{}); }
                        if (kb == 2) { if (i == 0) slot(std::integral_constant<int, 6>{}); if (i == 1) slot(std::integral_constant<int, 7>{}); if (i == 2) slot(std::integral_constant<int, 8>{}); }
                        if (kb == 3) { if (i == 0) slot(std::integral_constant<int, 9>{}); if (i == 1) slot(std::integral_constant<int, 10>{}); if (i == 2) slot(std::integral_constant<int, 11>{}); }
                    }
                }
                // A wave issues in order: while it waits to issue the next matrix instruction nothing else of it
                // issues.  So one matrix instruction (32 clocks in its pipe) is followed by up to seven vector
                // instructions (4 clocks each) and one LDS / memory instruction, 36 times.
                // The fragments of the next 16 positions are read in one go before the nine instructions that
                // hide their latency.
                __builtin_amdgcn_sched_group_barrier(0x100, 6, 0);          // LDS reads: fragments of block 0
#pragma unroll
                for (int kb = 0; kb < 4; ++kb) {
                    if (kb < 3) __builtin_amdgcn_sched_group_barrier(0x100, 6, 0);
#pragma unroll
                    for (int g = 0; g < 9; ++g) {
                        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // matrix
                        __builtin_amdgcn_sched_group_barrier(0x002, 7, 0);  // vector ALU
                        __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);  // LDS write
                    }
                }
                if (near_end(n, pn)) a_fix_tail(n, pn, buf ^ 1);
            } else {
#pragma unroll
                for (int kb = 0; kb < 4; ++kb) {
                    if (kb < nkb) {
                        if (kb + 1 < nkb) read((kb + 1) & 1, kb + 1);
#pragma unroll
                        for (int i = 0; i < 3; ++i)
#pragma unroll
                            for (int t = 0; t < 3; ++t)
                                acc[i][t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[kb & 1][i], fb[kb & 1][t],
                                                                                    acc[i][t], 0, 0, 0);
                    }
                }
                slot(std::integral_constant<int, 0>{}); slot(std::integral_constant<int, 1>{});
                slot(std::integral_constant<int, 2>{}); slot(std::integral_constant<int, 3>{});
                slot(std::integral_constant<int, 4>{}); slot(std::integral_constant<int, 5>{});
                slot(std::integral_constant<int, 6>{}); slot(std::integral_constant<int, 7>{});
                slot(std::integral_constant<int, 8>{}); slot(std::integral_constant<int, 9>{});
                slot(std::integral_constant<int, 10>{}); slot(std::integral_constant<int, 11>{});
                if (near_end(n, pn)) a_fix_tail(n, pn, buf ^ 1);
            }
            __syncthreads();
            buf ^= 1;
        };
        // (no way out of the loop between its three steps: an edge from there back to the loop head would carry
        // loads that were just issued, and the first register reuse at the head would wait for them)
        int prow = p_begin;
        for (; prow + 3 <= p_end; prow += 3) {
            step(std::integral_constant<int, 0>{}, prow);
            step(std::integral_constant<int, 1>{}, prow + 1);
            step(std::integral_constant<int, 2>{}, prow + 2);
        }
        if (prow < p_end) step(std::integral_constant<int, 0>{}, prow);
        if (prow + 1 < p_end) step(std::integral_constant<int, 1>{}, prow + 1);
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

// ---------------------------------------------------------------------------
// The same decomposition for fp32 tensors (v_mfma_f32_32x32x2_f32: one value per lane and operand, so no
// alignment question and no shifted copies): a work-group owns the whole K x (C*R*S) result for its (image,
// output-row range) units and walks the output rows.  Twelve waves, three per SIMD -- a wave that waits for its
// LDS reads or at the barrier leaves the matrix pipe to the other two --, each with the 96 rows x 32 taps of one
// column block in registers (3 blocks of 32 x 32).  Per output row p the LDS holds
//   xr[c][ring row][WP]   the input rows stride*p .. (fp32, zero padding columns in place, ring of 16 rows per
//                         channel; a step adds the `stride` rows the next output row needs)
//   dyr[buf][m][58]       dy(n, m, p, 0..Q-1), zero from Q on; pitch 58: the 64 lanes (m, k parity) of one read
//                         cover the 64 banks once
// and reduction pair t (positions 2t, 2t+1) costs four single-word LDS reads per wave -- three dy values, one
// input value at patch offset row*WP + stride*(2t + k) + s -- for three matrix instructions of 64 clocks, all
// with immediate offsets.  One output row is 9 * ceil(Q/2) matrix instructions per SIMD (16 k clocks for the
// first layer) against a few hundred clocks of staging, so the next row's loads simply sit in registers across
// the row.
// ---------------------------------------------------------------------------
constexpr int kRowsF32Threads = 768;
constexpr int kRowsF32DyPitch = 58;
constexpr int kRowsF32DyBuf = kRowsM * kRowsF32DyPitch;       // floats per dy buffer
constexpr int kRowsF32Slack = 64;                             // floats behind the input rows: reads one pair too far

struct WgradRowsF32Args {
    const float *x, *dy;
    float *part;                 // [work-group][K][Kg]
    int N, C, H, W, K, R, S, P, Q, Kg, stride, pad;
    int x_bs, y_bs;
    int splits, units;
    int WP;                      // LDS row pitch in floats: >= W + 2 * pad, = 48 mod 64
    int nnew;                    // input rows a step adds per channel: min(R, stride)
    FastDiv div_splits;
};

__global__ __launch_bounds__(kRowsF32Threads, 1) void wgrad_rows_f32_kernel(const WgradRowsF32Args p)
{
    extern __shared__ __attribute__((aligned(16))) float lds_fast[];
    float *const dyr = lds_fast;                               // two buffers
    float *const xr = lds_fast + 2 * kRowsF32DyBuf;
    const int tid = threadIdx.x, lane = tid & 63, wave = uniform(tid >> 6);
    const int l32 = lane & 31, half = lane >> 5;
    const int xchan = kRowsRing * p.WP;
    const int lds_floats = 2 * kRowsF32DyBuf + p.C * xchan + kRowsF32Slack;
    for (int o = tid; o < lds_floats; o += kRowsF32Threads) lds_fast[o] = 0.f;   // padding, positions >= Q: zero

    // this lane's tap: float offset of (c, ring row 0, column s + stride * k parity) and the filter row r
    int tap_off, tap_r;
    {
        const int j = 32 * wave + l32;
        const int jj = j < p.Kg ? j : 0;
        const int c = jj / (p.R * p.S), rs = jj - c * (p.R * p.S);
        const int r = rs / p.S, s = rs - r * p.S;
        tap_off = c * xchan + s + p.stride * half;
        tap_r = r;
    }

    f32x16 acc[3];
#pragma unroll
    for (int i = 0; i < 3; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;

    // Staging with addresses that cost nothing per element: thread t owns position q = t % 64 of the dy rows
    // m = t / 64 + 12u (u = 0..7) and column w = t % 256 of the new input rows (c, i) = slot t / 256 + 3v
    // (v = 0..5, slot = 4c + i); what changes from element to element is uniform.
    constexpr int NDY = kRowsM / 12;                           // 8 dy values per thread
    constexpr int NXR = 6;
    const int dq = tid & 63, dm = tid >> 6;
    const bool dq_on = dq < p.Q;
    const int xw = tid & 255, xs0 = tid >> 8;
    const int nfull = p.Q >> 1;                                // reduction pairs with both positions

    for (int unit = blockIdx.x; unit < p.units; unit += gridDim.x) {
        const int n = (int)fastdiv((uint32_t)unit, p.div_splits);
        const int sp = unit - n * p.splits;
        const int p_begin = (int)((int64_t)p.P * sp / p.splits), p_end = (int)((int64_t)p.P * (sp + 1) / p.splits);
        if (p_begin >= p_end) continue;
        const float *xn = p.x + (size_t)n * p.x_bs, *dyn = p.dy + (size_t)n * p.y_bs;
        __syncthreads();
        // input rows first_hh .. first_hh + rows - 1 (image row = hh - pad) of every channel; rows outside the
        // image are zero.  (Loads read a clamped, always valid address and nothing touches the value before the
        // matching store: a select on a loaded value would make the thread wait for each load in turn.)
        auto load_x = [&](float (&v)[NXR], int first_hh, int rows) {
            const int w = min(xw, p.W - 1);
#pragma unroll
            for (int u = 0; u < NXR; ++u) {
                const int slot = xs0 + 3 * u, c = slot >> 2, i = slot & 3;
                const int h = min(max(first_hh + i - p.pad, 0), p.H - 1);
                v[u] = xn[(min(c, p.C - 1) * p.H + h) * p.W + w];
            }
        };
        auto store_x = [&](const float (&v)[NXR], int first_hh, int rows) {
#pragma unroll
            for (int u = 0; u < NXR; ++u) {
                const int slot = xs0 + 3 * u, c = slot >> 2, i = slot & 3;
                if (c < p.C && i < rows && xw < p.W) {
                    const bool inside = (unsigned)(first_hh + i - p.pad) < (unsigned)p.H;
                    xr[c * xchan + ((first_hh + i) & (kRowsRing - 1)) * p.WP + p.pad + xw] = inside ? v[u] : 0.f;
                }
            }
        };
        auto load_dy = [&](float (&v)[NDY], int prow) {
            const float *src = dyn + prow * p.Q + min(dq, p.Q - 1);
#pragma unroll
            for (int u = 0; u < NDY; ++u) v[u] = src[min(dm + 12 * u, p.K - 1) * p.P * p.Q];
        };
        auto store_dy = [&](const float (&v)[NDY], int buf) {
            float *dst = dyr + buf * kRowsF32DyBuf + dm * kRowsF32DyPitch + dq;
            if (dq_on) {
#pragma unroll
                for (int u = 0; u < NDY; ++u)
                    if (dm + 12 * u < p.K) dst[12 * u * kRowsF32DyPitch] = v[u];
            }
        };
        float vx[NXR], vdy[NDY];
        // every input row of the first output row (R rows, in passes of nnew), and its dy row
        for (int r0 = 0; r0 < p.R; r0 += p.nnew) {
            const int rows = min(p.nnew, p.R - r0);
            load_x(vx, p.stride * p_begin + r0, rows);
            store_x(vx, p.stride * p_begin + r0, rows);
        }
        load_dy(vdy, p_begin);
        store_dy(vdy, 0);
        __syncthreads();
        int buf = 0;
        for (int prow = p_begin; prow < p_end; ++prow) {
            const bool more = prow + 1 < p_end;
            const int hh_new = p.stride * (prow + 1) + p.R - p.nnew;
            if (more) {
                load_x(vx, hh_new, p.nnew);
                load_dy(vdy, prow + 1);
            }
            const float *Ab = dyr + buf * kRowsF32DyBuf + l32 * kRowsF32DyPitch + half;
            const float *Bb = xr + tap_off + ((p.stride * prow + tap_r) & (kRowsRing - 1)) * p.WP;
            float fa[2][3], fb[2];
            // operands of pair tp; a pair past the last one may be read (never used): the reads stay inside LDS
            auto read = [&](int set, int tp) {
#pragma unroll
                for (int i = 0; i < 3; ++i) fa[set][i] = Ab[i * 32 * kRowsF32DyPitch + 2 * tp];
                fb[set] = Bb[2 * p.stride * tp];
            };
            auto mfmas = [&](int set) {
#pragma unroll
                for (int i = 0; i < 3; ++i)
                    acc[i] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[set][i], fb[set], acc[i], 0, 0, 0);
            };
            read(0, 0);
            int tp = 0;
            // no branch inside (the waits count the reads), and the order is pinned: the reads of the next pair
            // are issued before this pair's matrix instructions
            for (; tp + 2 <= nfull; tp += 2) {
                read(1, tp + 1);
                __builtin_amdgcn_sched_barrier(0);
                mfmas(0);
                __builtin_amdgcn_sched_barrier(0);
                read(0, tp + 2);
                __builtin_amdgcn_sched_barrier(0);
                mfmas(1);
                __builtin_amdgcn_sched_barrier(0);
            }
            if (tp < nfull) {                                   // set 0 holds pair tp
                if (p.Q & 1) read(1, tp + 1);
                mfmas(0);
                ++tp;
                if (p.Q & 1) {
                    // last position alone: the missing odd position reads dy's zero at Q and, for the input, that
                    // same zero word, so that no input value is multiplied by it
                    if (half) fb[1] = fa[1][0];
                    mfmas(1);
                }
            } else if (p.Q & 1) {                               // set 0 holds the half pair nfull
                if (half) fb[0] = fa[0][0];
                mfmas(0);
            }
            if (more) {
                store_x(vx, hh_new, p.nnew);
                store_dy(vdy, buf ^ 1);
            }
            __syncthreads();
            buf ^= 1;
        }
    }

    float *out = p.part + (size_t)blockIdx.x * p.K * p.Kg;
    const int col = 32 * wave + l32;
#pragma unroll
    for (int i = 0; i < 3; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int row = 32 * i + (v >> 2) * 8 + half * 4 + (v & 3);
            if (row < p.K && col < p.Kg) out[(size_t)row * p.Kg + col] = acc[i][v];
        }
}
