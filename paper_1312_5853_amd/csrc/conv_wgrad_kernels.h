// Backward-filter kernels (tap table, fast, bf16, bf16 linear) and the kernels that sum their partials.
// Part of convnet_hotpath.hip: included there, inside its anonymous namespace, after the common
// definitions (kThreads, kPitch, vector types); not a stand-alone header.
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
// The x loads are 4-byte aligned: xp is kept twice, the second copy moved up by one element for the odd tap shifts.
// Columns in (r, s, c) order, partials [split][K][R*S*C] as in wgrad_fast_kernel.
// ---------------------------------------------------------------------------
// ---------------------------------------------------------------------------
// The kernel: both operands are loaded from global memory straight into LDS (16 bytes per lane, no staging
// registers and no LDS store instructions: at bf16 matrix rates the 32 KB a 128 x 128 tile stores into LDS per
// 64-position step take as long as its matrix work, see conv_bf16_dma_kernels.h).  One eight-wave work-group per
// CU owns a 128 x 256 tile (rows: filters, columns: taps (r, s, c)) for a range of the reduction; three LDS buffers
// of (128 + 256) rows of 64 positions = 48 KB each; the loads of step s + 2 are in flight while step s is multiplied.
// Operand layouts (pack_lin):
//   dyT[step][Kpad][64]   dy with the zero padding in place as in dyp, but step-major, and the eight 16-byte chunks of
//                         a row stored at position chunk ^ swz(row), swz(row) = (row >> 1) & 7: a step's 128 rows are
//                         one contiguous 16 KB block that is copied linearly, and the 16 lanes of a fragment read
//                         cover the 64 banks
//   xp                    as above (two copies); lane (row, slot) of a load fetches chunk slot ^ swz(row) of its column's
//                         row, so the LDS rows come out swizzled the same way
// ---------------------------------------------------------------------------
struct WgradLinDmaArgs {
    const unsigned short *dyT;
    const unsigned short *xp;
    float *part;
    int K, Kpad, C, ncols;
    int S, Wq;
    int N, G, Jx;             // G = Jy / 8 groups of 8 positions per image
    int row_x_bytes;          // bytes per xp row (N * Jx * 2)
    int steps, steps_per_split;
    int mtiles, ntiles, nunits, units_per_xcd;
    FastDiv div_c, div_s, div_g;
};

template <int TM, int TN, int WM, int WN>
__global__ __launch_bounds__(WM * WN * 64, 1) void wgrad_bf16_lin_dma_kernel(const WgradLinDmaArgs p)
{
    constexpr int NT = WM * WN * 64;
    constexpr int BM = TM * WM * 32, BN = TN * WN * 32;
    constexpr int RB = 128, CH = 8, NK = 4;              // 64 positions per row and step
    constexpr int NA = BM * CH / NT, NB = BN * CH / NT, NL = NA + NB;
    constexpr int BUF = (BM + BN) * RB;
    static_assert((BM * CH) % NT == 0 && (BN * CH) % NT == 0, "whole wavefront loads");
    static_assert(NB % 2 == 0, "a thread's loads alternate between two chunks");

    extern __shared__ __attribute__((aligned(16))) float lds_fast[];
    const char *const lds = reinterpret_cast<const char *>(lds_fast);
    const unsigned lds_base = (unsigned)(size_t)lds_fast;

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

    const int step_begin = split * p.steps_per_split;
    const int nsteps = min(p.steps - step_begin, p.steps_per_split);

    // x loads: load u of this thread fills chunk slot (lane % 8) of tile row (wave*NB + u)*8 + lane / 8 with chunk
    // slot ^ swz(row) of that column's row; swz(row) = (lane / 16 + 4 * ((wave*NB + u) & 1)) & 7, so a thread's loads
    // alternate between two chunks (u even / odd), each with its own (image, group) position that moves on by 8 groups
    // per step
    unsigned bbase[NB];
    const int slot = lane & 7;
#pragma unroll
    for (int u = 0; u < NB; ++u) {
        const int row = (wave * NB + u) * 8 + (lane >> 3);
        int col = n0 + row;
        col = col < p.ncols ? col : 0;
        const int rs = (int)fastdiv((uint32_t)col, p.div_c), c = col - rs * p.C;
        const int r = (int)fastdiv((uint32_t)rs, p.div_s), sx = rs - r * p.S;
        const int shift = r * p.Wq + sx;                   // odd shifts read the copy that is moved up by one element
        bbase[u] = (uint32_t)(c + (shift & 1) * p.C) * (uint32_t)p.row_x_bytes + 2u * (uint32_t)(shift & ~1);
    }
    int pn[2], pg[2];
#pragma unroll
    for (int e = 0; e < 2; ++e) {
        const int chunk = slot ^ (((lane >> 4) + 4 * ((wave * NB + e) & 1)) & 7);
        const int g = step_begin * 8 + chunk;
        pn[e] = (int)fastdiv((uint32_t)g, p.div_g);
        pg[e] = g - pn[e] * p.G;
    }
    const unsigned aoff = (unsigned)((wave * NA * 64 + lane) * 16);
    const size_t a_step_bytes = (size_t)p.Kpad * RB;
    const char *a_base = reinterpret_cast<const char *>(p.dyT) + (size_t)step_begin * a_step_bytes + (size_t)m0 * RB;
    const char *const xpb = reinterpret_cast<const char *>(p.xp);

    unsigned la = 0, lb = 0, pos[2] = {0u, 0u};
    auto begin_step_loads = [&](int buf) {
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            pos[e] = 2u * (unsigned)(min(pn[e], p.N - 1) * p.Jx + pg[e] * 8);   // steps past the last image: zero dy
            pg[e] += 8;
            const bool wrap = pg[e] >= p.G;
            pg[e] -= wrap ? p.G : 0;
            pn[e] += wrap ? 1 : 0;
        }
        la = lds_base + buf * BUF + wave * NA * 1024;
        lb = lds_base + buf * BUF + BM * RB + wave * NB * 1024;
    };
    auto load_one = [&](int i) {     // i < NL, compile-time after unrolling
        if (i < NA) dma16(a_base, aoff + i * 1024, la + i * 1024);
        else dma16(xpb, bbase[i - NA] + pos[(i - NA) & 1], lb + (i - NA) * 1024);
    };
    auto end_step_loads = [&]() { a_base += a_step_bytes; };
    auto load_step = [&](int buf) {
        begin_step_loads(buf);
#pragma unroll
        for (int i = 0; i < NL; ++i) load_one(i);
        end_step_loads();
    };

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int jn = 0; jn < TN; ++jn)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][jn][v] = 0.f;

    const int l32 = lane & 31, half = lane >> 5;
    const int swzl = (l32 >> 1) & 7;
    int koff[NK];
#pragma unroll
    for (int t = 0; t < NK; ++t) koff[t] = ((2 * t + half) ^ swzl) * 16;
    const int a_row = (wm * TM * 32 + l32) * RB;
    const int b_row = BM * RB + (wn * TN * 32 + l32) * RB;

    u32x4 fa[2][TM], fb[2][TN];
    auto read_frags = [&](const char *bufp, int t, int set) {
#pragma unroll
        for (int i = 0; i < TM; ++i) fa[set][i] = *reinterpret_cast<const u32x4 *>(bufp + a_row + i * 32 * RB + koff[t]);
#pragma unroll
        for (int jn = 0; jn < TN; ++jn) fb[set][jn] = *reinterpret_cast<const u32x4 *>(bufp + b_row + jn * 32 * RB + koff[t]);
    };

    if (nsteps > 0) load_step(0);
    if (nsteps > 1) load_step(1);
    if (nsteps > 1) wait_vmcnt<NL>(); else wait_vmcnt<0>();
    __syncthreads();
    if (nsteps > 0) read_frags(lds, 0, 0);

    // One step: see colgemm_bf16_dma_kernel (slices of 16 positions, the loads of step + 2 spread over slices
    // 0 .. NK-2, the barrier before the last slice, slice 0 of the next step read behind it).
    constexpr int MPS = TM * TN;
    constexpr int SLOTS = (NK - 1) * MPS;
    constexpr int SPACING = SLOTS / NL > 0 ? SLOTS / NL : 1;
    static_assert(NL <= SLOTS, "one load per matrix instruction at most");
    int step = 0;
    auto do_step = [&](auto more_c) {
        constexpr bool more = decltype(more_c)::value;
        const char *bufp = lds + (step % 3) * BUF;
        const char *nextp = lds + ((step + 1) % 3) * BUF;
        if (more) begin_step_loads((step + 2) % 3);
#pragma unroll
        for (int t = 0; t < NK; ++t) {
            if (t + 1 < NK) {
                read_frags(bufp, t + 1, (t + 1) & 1);
            } else {
                if (more) wait_vmcnt<NL>(); else wait_vmcnt<0>();
                asm volatile("s_waitcnt lgkmcnt(0)");
                __syncthreads();
                if (more || step + 1 < nsteps) read_frags(nextp, 0, (t + 1) & 1);
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int jn = 0; jn < TN; ++jn) {
                    acc[i][jn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fa[t & 1][i]),
                                                                         __builtin_bit_cast(bf16x8, fb[t & 1][jn]),
                                                                         acc[i][jn], 0, 0, 0);
                    const int m = t * MPS + i * TN + jn;
                    if (more && t + 1 < NK && m % SPACING == SPACING - 1 && m / SPACING < NL) {
                        __builtin_amdgcn_sched_barrier(0);
                        load_one(m / SPACING);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
            __builtin_amdgcn_sched_barrier(0);
        }
        if (more) end_step_loads();
        ++step;
    };
    while (step + 2 < nsteps) do_step(std::true_type{});
    while (step < nsteps) do_step(std::false_type{});

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

// dyp[k][e], e < row_elems: image n = e / Jy, j = e % Jy = p*Wq + q; dy(n, k, p, q) where p < P and q < Q, else 0.
// One thread per 8 consecutive elements (Jy and row_elems are multiples of 8, so they share k and n): eight
// 2-byte loads along a row of dy, one 16-byte store.
__device__ __forceinline__ void pack_dy_lin(int64_t i8, const unsigned short *__restrict__ dy,
                                            unsigned short *__restrict__ dyp, int N, int K, int P, int Q, int Wq, int Jy,
                                            int row_elems, int64_t dy_bs, FastDiv div_row, FastDiv div_jy,
                                            FastDiv div_wq, int kpad)
{
    const int64_t i = i8 * 8;
    if (i >= (int64_t)K * row_elems) return;
    const uint32_t k = fastdiv((uint32_t)i, div_row), e = (uint32_t)i - k * (uint32_t)row_elems;
    const uint32_t n = fastdiv(e, div_jy), j = e - n * (uint32_t)Jy;
    uint32_t pp = fastdiv(j, div_wq), q = j - pp * (uint32_t)Wq;
    const unsigned short *src = dy + n * dy_bs + (int64_t)k * P * Q;
    unsigned short v[8];
#pragma unroll
    for (int t = 0; t < 8; ++t) {
        v[t] = (n < (uint32_t)N && pp < (uint32_t)P && q < (uint32_t)Q) ? src[pp * Q + q] : (unsigned short)0;
        if (++q == (uint32_t)Wq) { q = 0; ++pp; }
    }
    u32x4 o = {(uint32_t)v[0] | (uint32_t)v[1] << 16, (uint32_t)v[2] | (uint32_t)v[3] << 16,
               (uint32_t)v[4] | (uint32_t)v[5] << 16, (uint32_t)v[6] | (uint32_t)v[7] << 16};
    if (kpad == 0) {
        reinterpret_cast<u32x4 *>(dyp)[i8] = o;
    } else {
        // dyT[step][Kpad][64]: chunk (e % 64) / 8 of row k and step e / 64 goes to position chunk ^ swz(k)
        const uint32_t st = e >> 6, chunk = (e >> 3) & 7;
        reinterpret_cast<u32x4 *>(dyp)[((size_t)st * kpad + k) * 8 + (chunk ^ ((k >> 1) & 7))] = o;
    }
}

// xp[c][n][e], e < Jx: padded row hh = e / Wq, column ww = e % Wq; x(n, c, hh - pad, ww - pad) where inside, else 0.
// One thread per 8 consecutive elements (Jx is a multiple of 8).  A second copy follows the first, moved up by one
// element (copy 1 at e holds copy 0 at e + 1, zero at the end of a row): a tap with an odd shift reads it at shift - 1,
// so that every operand load of the main kernel is 4-byte aligned -- 16-byte loads from addresses that are only 2-byte
// aligned run at a quarter of the rate on this chip.
__device__ __forceinline__ void pack_x_lin(int64_t i8, const unsigned short *__restrict__ x,
                                           unsigned short *__restrict__ xp, int N, int C, int H, int W, int pad, int Wq,
                                           int Jx, int64_t x_bs, FastDiv div_jx, FastDiv div_wq)
{
    const int64_t i = i8 * 8;
    if (i >= (int64_t)C * N * Jx) return;
    const uint32_t cn = fastdiv((uint32_t)i, div_jx), e = (uint32_t)i - cn * (uint32_t)Jx;
    const uint32_t c = cn / (uint32_t)N, n = cn - c * (uint32_t)N;
    uint32_t hh = fastdiv(e, div_wq), ww = e - hh * (uint32_t)Wq;
    const unsigned short *src = x + n * x_bs + (int64_t)c * H * W;
    unsigned short v[9];
#pragma unroll
    for (int t = 0; t < 9; ++t) {
        const int h = (int)hh - pad, w = (int)ww - pad;
        v[t] = (e + t < (uint32_t)Jx && (unsigned)h < (unsigned)H && (unsigned)w < (unsigned)W) ? src[h * W + w]
                                                                                                 : (unsigned short)0;
        if (++ww == (uint32_t)Wq) { ww = 0; ++hh; }
    }
    u32x4 o = {(uint32_t)v[0] | (uint32_t)v[1] << 16, (uint32_t)v[2] | (uint32_t)v[3] << 16,
               (uint32_t)v[4] | (uint32_t)v[5] << 16, (uint32_t)v[6] | (uint32_t)v[7] << 16};
    reinterpret_cast<u32x4 *>(xp)[i8] = o;
    u32x4 o1 = {(uint32_t)v[1] | (uint32_t)v[2] << 16, (uint32_t)v[3] | (uint32_t)v[4] << 16,
                (uint32_t)v[5] | (uint32_t)v[6] << 16, (uint32_t)v[7] | (uint32_t)v[8] << 16};
    reinterpret_cast<u32x4 *>(xp + (int64_t)C * N * Jx)[i8] = o1;
}

// Both packing passes in one launch: blocks [0, dy_blocks) pack dy, the rest pack x.
struct PackLinArgs {
    const unsigned short *dy, *x;
    unsigned short *dyp, *xp;
    int N, K, C, P, Q, H, W, pad, Wq, Jy, Jx, row_elems, dy_blocks;
    int kpad;              // > 0: dy goes to the step-major swizzled layout dyT[step][kpad][64] (rows K..kpad-1 are not
                           // written: what the kernel computes from them is never stored)
    int64_t dy_bs, x_bs;
    FastDiv div_row, div_jy, div_jx, div_wq;
};

__global__ __launch_bounds__(256) void pack_lin(const PackLinArgs a)
{
    if ((int)blockIdx.x < a.dy_blocks)
        pack_dy_lin((int64_t)blockIdx.x * 256 + threadIdx.x, a.dy, a.dyp, a.N, a.K, a.P, a.Q, a.Wq, a.Jy, a.row_elems,
                    a.dy_bs, a.div_row, a.div_jy, a.div_wq, a.kpad);
    else
        pack_x_lin((int64_t)(blockIdx.x - a.dy_blocks) * 256 + threadIdx.x, a.x, a.xp, a.N, a.C, a.H, a.W, a.pad, a.Wq,
                   a.Jx, a.x_bs, a.div_jx, a.div_wq);
}

// dw[k][c][rs] = part[0][k][rs*C + c] + part[1][k][rs*C + c] + ...  (fixed order)
// groups > 1: K filters per column; the partials of column g follow those of column g - 1, dw holds the columns'
// filters one after the other
// (one thread per output word: a thread per (k, c) plane that loops over the taps and splits reads and writes
// better-shaped runs but has 54 dependent loads in a row and was 4-10 times slower)
__global__ void finish_wgrad(const float *__restrict__ part, float *__restrict__ dw, int K, int C, int RS,
                             int nsplit, int groups, FastDiv div_kcols, FastDiv div_cols, FastDiv div_c)
{
    const int ncols = RS * C;
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= groups * K * ncols) return;
    const int gcol = (int)fastdiv((uint32_t)i, div_kcols);
    i -= gcol * (K * ncols);
    part += (size_t)gcol * nsplit * K * ncols;
    dw += (size_t)gcol * K * ncols;
    const int k = (int)fastdiv((uint32_t)i, div_cols), col = i - k * ncols;
    const int rs = (int)fastdiv((uint32_t)col, div_c), c = col - rs * C;
    float s = part[i];
    for (int t = 1; t < nsplit; ++t) s += part[(size_t)t * K * ncols + i];
    dw[((size_t)k * C + c) * RS + rs] = s;
}

// The same for a channel count that is a multiple of four: a thread adds four consecutive columns (one tap, four
// channels) of all splits with 16-byte loads, in the same order as above, and stores the four words.
__global__ __launch_bounds__(256) void finish_wgrad_x4(const float *__restrict__ part, float *__restrict__ dw, int K,
                                                        int C, int RS, int nsplit, int groups, FastDiv div_kquads,
                                                        FastDiv div_quads, FastDiv div_c)
{
    const int ncols = RS * C, nquads = ncols / 4;
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= groups * K * nquads) return;
    const int gcol = (int)fastdiv((uint32_t)i, div_kquads);
    i -= gcol * (K * nquads);
    part += (size_t)gcol * nsplit * K * ncols;
    dw += (size_t)gcol * K * ncols;
    const int k = (int)fastdiv((uint32_t)i, div_quads), col = 4 * (i - k * nquads);
    const int rs = (int)fastdiv((uint32_t)col, div_c), c = col - rs * C;
    const f32x4 *src = reinterpret_cast<const f32x4 *>(part + (size_t)k * ncols + col);
    const size_t split_quads = (size_t)K * nquads;
    f32x4 s = src[0];
#pragma unroll 4
    for (int t = 1; t < nsplit; ++t) s += src[t * split_quads];
    float *out = dw + ((size_t)k * C + c) * RS + rs;
    out[0] = s[0]; out[RS] = s[1]; out[2 * RS] = s[2]; out[3 * RS] = s[3];
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

// The same for many partials and a count that is a multiple of four (16-byte aligned dw): four consecutive outputs
// per thread, 16 lane groups; group g adds the partials g, g + 16, g + 32, ... in ascending order, then the sixteen
// sums are added in group order.
__global__ __launch_bounds__(256) void reduce_partials_x4(const float *__restrict__ part, float *__restrict__ dw,
                                                           int count, int nsplit)
{
    __shared__ f32x4 sums[16][16];
    const int o = threadIdx.x & 15, g = threadIdx.x >> 4;
    const int i = (blockIdx.x * 16 + o) * 4;
    f32x4 s = {0.f, 0.f, 0.f, 0.f};
    if (i < count)
        for (int k = g; k < nsplit; k += 16) s += *reinterpret_cast<const f32x4 *>(part + (size_t)k * count + i);
    sums[g][o] = s;
    __syncthreads();
    if (g == 0 && i < count) {
        f32x4 t = sums[0][o];
        for (int q = 1; q < 16; ++q) t += sums[q][o];
        *reinterpret_cast<f32x4 *>(dw + i) = t;
    }
}
