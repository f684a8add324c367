// Forward / backward-data kernels (tap table, fast, 48-row, bf16, patch) and their helper kernels.
// Part of convnet_hotpath.hip: included there, inside its anonymous namespace, after the common
// definitions (kThreads, kPitch, vector types); not a stand-alone header.
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
    int64_t src_gb, dst_gb, at_gb;      // the same strides in bytes, for the bf16 kernel (bf16 copies, bf16 or fp32 dst)
    // applied where the final sums are stored (this kernel when ksplit == 1 and epi_on, else the split-sum kernel)
    int epi_on;
    Epilogue epi;
    FastDiv div_plane, div_ow, div_rs, div_s;
};

// KC = reduction depth of one step (16 or 32 channels of one tap).  LDS is
// dynamic: 2 * (BM + BN) * (KC + 4) floats.
template <int TM, int TN, int WM, int WN, int KC>
__global__ __launch_bounds__(kThreads, (TM == 3 && TN == 1) ? 3 : 2) void colgemm_fast_kernel(const ColGemmFastArgs p)
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

    load_step(0);
    store_step(0);
    if (nsteps > 1) load_step(1);
    __syncthreads();
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
    if (idx >= p.tiles_per_xcd || unit >= ntile * p.ksplit * p.groups) return;
    const int grp_col = unit / (ntile * p.ksplit);              // column of a grouped layer
    const int unit_c = unit - grp_col * (ntile * p.ksplit);
    const int ks = unit_c / ntile;
    const int tile = unit_c - ks * ntile;
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
    const char *src_bytes = reinterpret_cast<const char *>(p.src) + (size_t)grp_col * p.src_gb;
    const size_t a_step = (size_t)p.Mpad * (KC / 8);          // 16-byte vectors per step
    const int step_begin = ks * p.steps_per_split;
    const int nsteps = min(p.cblocks * p.R * p.S - step_begin, p.steps_per_split);
    const u32x4 *a_ptr = reinterpret_cast<const u32x4 *>(reinterpret_cast<const char *>(p.At) + (size_t)grp_col * p.at_gb) +
                         (size_t)m0 * (KC / 8) + tid + step_begin * a_step;

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
            unsigned short *out = reinterpret_cast<unsigned short *>(reinterpret_cast<char *>(p.dst) + (size_t)grp_col * p.dst_gb) +
                                  (size_t)n * p.dst_bs + rem;
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
        float *out = p.ksplit > 1
                         ? p.part + (size_t)grp_col * p.part_gs + ((size_t)ks * (p.ncols / plane) + n) * ((size_t)p.M * plane) + rem
                         : reinterpret_cast<float *>(reinterpret_cast<char *>(p.dst) + (size_t)grp_col * p.dst_gb) +
                               (size_t)n * p.dst_bs + rem;
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

// bf16 filters for colgemm_bf16_kernel: wt[((cb*R + r)*S + s)][Mpad][kc]; groups > 1: the filters of column g
// start w_gs elements after those of column g - 1, the copies are consecutive
__global__ void relayout_filters_cblk_bf16(const unsigned short *__restrict__ w, unsigned short *__restrict__ wt,
                                           int M, int Mpad, int cblocks, int RS, int C, int transposed, int kc,
                                           int groups, int64_t w_gs)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t total = (int64_t)cblocks * RS * Mpad * kc;
    if (i >= total * groups) return;
    const int64_t gcol = i / total;
    w += gcol * w_gs;
    wt += gcol * total;
    i -= gcol * total;
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

// The same re-layout with one thread per four consecutive channels (one 16-byte store) and 32-bit index arithmetic
// with precomputed divisions: the launch is short (a few MB), so the per-element 64-bit divisions above were most of it.
// Needs fewer than 2^31 elements in all.
__global__ void relayout_filters_cblk_x4(const float *__restrict__ w, float *__restrict__ wt, int M, int Mpad,
                                         int cblocks, int RS, int C, int transposed, int kc, int groups, int64_t w_gs,
                                         FastDiv div_mpad, FastDiv div_rs, FastDiv div_cb)
{
    const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    const uint32_t quads = (uint32_t)kc / 4;                        // 4 or 8
    const uint32_t total = (uint32_t)groups * cblocks * RS * Mpad * quads;
    if (i >= total) return;
    const uint32_t q = i & (quads - 1), t0 = i / quads;             // (a shift: quads is a power of two)
    const uint32_t t1 = fastdiv(t0, div_mpad), m = t0 - t1 * (uint32_t)Mpad;
    const uint32_t t2 = fastdiv(t1, div_rs), rs = t1 - t2 * (uint32_t)RS;       // t2 = gcol * cblocks + cb
    const uint32_t gcol = fastdiv(t2, div_cb), cb = t2 - gcol * (uint32_t)cblocks;
    const float *wg = w + gcol * w_gs;
    const uint32_t ch = cb * (uint32_t)kc + 4 * q;
    f32x4 v = {0.f, 0.f, 0.f, 0.f};
    if (m < (uint32_t)M) {
        const int64_t base = transposed ? ((int64_t)ch * C + m) * RS + rs : ((int64_t)m * C + ch) * RS + rs;
        const int64_t stride = transposed ? (int64_t)C * RS : RS;
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = wg[base + e * stride];
    }
    reinterpret_cast<f32x4 *>(wt)[i] = v;
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
    int epi_on;           // bias / ReLU applied to each fp32 sum before it is stored (and, for TO = bfloat16, rounded)
    int vec;              // fp32 rows staged in 16-byte pieces: W % 4 == 0, pad even, images 16-byte aligned
    Epilogue epi;
    FastDiv div_q, div_rs, div_s, div_mj, div_m, div_wp, div_nr, div_pr;   // div_pr: W / 4 pieces per staged row
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
        const TI *xn = static_cast<const TI *>(p.x) + (size_t)n * p.x_bs;
        const int total = p.vec ? 0 : p.C * p.NR * p.WP;
        if (sizeof(TI) == 4 && p.vec) {
            // 16-byte pieces of the image rows; sixteen loads in flight per thread (the first layer's patch is one
            // batch).  Rows outside the image are loaded from a valid address and zeroed when they are stored: a
            // select on the loaded value would wait for the load.  The store loop has one test per piece and no
            // inner loops; the pad columns are zeroed by a pass of their own.
            const float *xf = reinterpret_cast<const float *>(xn);
            const int pr = p.W >> 2, pieces = p.C * p.NR * pr;
            for (int e0 = tid; e0 < pieces; e0 += kThreads * 16) {
                f32x4 tmp[16];
                int dst[16];
                bool inside[16];
#pragma unroll
                for (int u = 0; u < 16; ++u) {
                    const int e = e0 + u * kThreads;
                    const int ee = e < pieces ? e : 0;
                    const int row = (int)fastdiv((uint32_t)ee, p.div_pr);
                    const int pc = ee - row * pr;
                    const int c = (int)fastdiv((uint32_t)row, p.div_nr);
                    const int h = h0 + row - c * p.NR;
                    const bool ok = (unsigned)h < (unsigned)p.H;
                    tmp[u] = *reinterpret_cast<const f32x4 *>(xf + (ok ? (c * p.H + h) * p.W + pc * 4 : 0));
                    inside[u] = ok;
                    dst[u] = e < pieces ? row * p.WP + p.pad + pc * 4 : -1;
                }
                typedef float f32x2 __attribute__((ext_vector_type(2)));
#pragma unroll
                for (int u = 0; u < 16; ++u) {
                    if (dst[u] >= 0) {                         // patch rows and pad are even: 8-byte stores
                        f32x2 *q = reinterpret_cast<f32x2 *>(&patch[dst[u]]);
                        q[0] = inside[u] ? f32x2{tmp[u][0], tmp[u][1]} : f32x2{0.f, 0.f};
                        q[1] = inside[u] ? f32x2{tmp[u][2], tmp[u][3]} : f32x2{0.f, 0.f};
                    }
                }
            }
            for (int r = tid; r < p.C * p.NR; r += kThreads) {
                typedef float f32x2 __attribute__((ext_vector_type(2)));
                float *rowp = &patch[r * p.WP];
                for (int v = 0; v < p.pad; v += 2) *reinterpret_cast<f32x2 *>(&rowp[v]) = f32x2{0.f, 0.f};
                for (int v = p.pad + p.W; v < p.WP; v += 2) *reinterpret_cast<f32x2 *>(&rowp[v]) = f32x2{0.f, 0.f};
            }
        }
        // any other shape or type, one value at a time: 32 independent loads in flight per thread and batch
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
        if (p.epi_on) {                                          // forward only: bias and ReLU, no mask
            float bv16[16];
#pragma unroll
            for (int v = 0; v < 16; ++v)
                bv16[v] = p.epi.bias ? p.epi.bias[min(row0 + (v >> 2) * 8 + (v & 3), p.M - 1)] : 0.f;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const float t = acc[i][v] + bv16[v];
                acc[i][v] = (p.epi.relu && !(t > 0.f)) ? 0.f : t;
            }
        }
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int row = row0 + (v >> 2) * 8 + (v & 3);
            if (row < p.M) st_elem(out, (int64_t)row * p.PQ, acc[i][v]);
        }
    }
}
