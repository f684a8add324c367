// Forward / stride-1 backward-data with bf16 inputs, second generation: both operands go from global memory
// straight into LDS (16 bytes per lane, no staging registers, no LDS store instructions).
// Part of convnet_hotpath.hip: included there, inside its anonymous namespace, after conv_colgemm_kernels.h.
//
// Why: on gfx950 an LDS store instruction moves about 75 bytes per clock and CU (ds_write_b128: 13.5 clocks per
// wavefront instruction) against 256 bytes per clock for ds_read_b128, and the vector memory path delivers 64 bytes
// per clock and CU.  At bf16 matrix rates (one 32x32x16 instruction = 32 clocks) a 128 x 128 tile staged through
// registers needs more LDS store time than matrix time.  Direct loads cost the memory path only, and a 128 x 256
// tile brings 48 KB per 64-channel step through it in 768 clocks against 1024 clocks of matrix work.
//
// Layouts the two preparation kernels below write into the workspace:
//   xb  activations, channel-blocked AND zero-padded: [n][channel block of 16][Hp][Wp][16 channels], 32 bytes per
//       position and block.  With the padding in place a filter tap is a constant address offset: no bounds
//       tests and no zero substitution remain in the main loop (a direct load could not substitute a zero).
//       Padded row of output row oh under tap r:  oh*mul + r (forward, pad rows above = pad) or oh + (R-1-r)
//       (backward-data, pad rows above = R-1-pad); columns alike.
//   wt  filters [step = (channel block of KC, r, s)][Mpad rows][KC channels], the eight-channel (16-byte) chunks of
//       a row stored at position chunk ^ swz(row): a linear copy into LDS then yields rows whose chunks are
//       XOR-swizzled, and the 16 lanes of one ds_read_b128 phase (16 rows, one chunk each) cover all 64 banks.
//       swz(row) = (row >> log2(256 / row bytes)) & (chunks - 1).
// LDS: three buffers of (BM + BN) rows of KC bf16 (unpadded rows: a wavefront's direct load fills 1 KB
// linearly).  Step s is multiplied out of buffer s % 3 while the loads of step s + 2 are in flight into the buffer
// that step s - 1 used; before the barrier that ends step s every wave waits until its loads of step s + 1 have
// landed (s_waitcnt vmcnt(loads per step)).
struct ColGemmDmaArgs {
    const void *At;        // wt (see above)
    const void *xb;        // blocked, padded activations
    void *dst;             // y or dx: fp32, or bfloat16 when out_bf16
    float *part;           // ksplit > 1: partial outputs [ksplit][N][M][OH*OW]
    int M, Mpad, ncols;
    int OH, OW, mul;
    int Wp;                // padded row pitch of xb in positions
    int cb_bytes;          // bytes of one (sample, channel block): Hp * Wp * 32
    int n_bytes;           // bytes of one sample: (channels / 16) * cb_bytes
    int R, S, sign;        // sign +1: tap (r, s) reads padded (oh*mul + r, ow*mul + s); -1: (oh + R-1-r, ow + S-1-s)
    int cblocks;           // channels / KC
    int dst_bs, out_bf16;
    int dst_small;         // a bfloat16 dst is shorter than 2 GB: byte offsets into it fit 32 bits
    int mtiles, ntiles, tiles_per_xcd, ksplit, steps_per_split;
    int epi_on;
    Epilogue epi;
    FastDiv div_plane, div_ow, div_rs, div_s;
};

// 16 bytes per lane from global memory (sbase + voff, voff per lane) into LDS at lds_base + lane * 16
// (lds_base wave-uniform, in bytes).  Counts on vmcnt like any vector memory load.  M0 (the LDS base of such loads)
// is set inside the statement; the compiler keeps no value of its own in that register across statements.
__device__ __forceinline__ void dma16(const void *sbase, unsigned voff, unsigned lds_base)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :: "s"(lds_base), "v"(voff), "s"(sbase));
}
template <int N>
__device__ __forceinline__ void wait_vmcnt() { asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N)); }

template <int TM, int TN, int WM, int WN, int KC, int OCC>
__global__ __launch_bounds__(WM * WN * 64, OCC) void colgemm_bf16_dma_kernel(const ColGemmDmaArgs p)
{
    constexpr int NT = WM * WN * 64;           // threads: four or eight waves
    constexpr int BM = TM * WM * 32, BN = TN * WN * 32;
    constexpr int RB = KC * 2;                 // bytes per LDS row
    constexpr int CH = KC / 8;                 // 16-byte chunks per row
    constexpr int SH = KC == 64 ? 1 : 2;       // log2(256 / RB)
    constexpr int NK = KC / 16;                // matrix instructions per 32 x 32 block and step
    constexpr int NA = BM * CH / NT;     // direct loads per thread and step: filters
    constexpr int NB = BN * CH / NT;     // ... activations
    constexpr int NL = NA + NB;
    constexpr int BUF = (BM + BN) * RB;        // bytes per LDS buffer
    static_assert(WM * WN == 4 || WM * WN == 8, "four or eight waves per work-group");
    static_assert(KC == 64 || KC == 32, "step depth");
    static_assert(NK % 2 == 0, "slice 0 of the next step lands in fragment set 0");
    static_assert((BM * CH) % NT == 0 && (BN * CH) % NT == 0, "whole wavefront loads");

    extern __shared__ __attribute__((aligned(16))) float lds_fast[];
    const char *const lds = reinterpret_cast<const char *>(lds_fast);
    const unsigned lds_base = (unsigned)(size_t)lds_fast;       // LDS byte address of buffer 0

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

    // --- activation loads: load u of this thread fills chunk slot (q % CH) of tile row q / CH, q = (wave*NB + u)*64 + lane,
    // with the chunk (slot ^ swz(row)) of that row's position
    unsigned boff[NB];
#pragma unroll
    for (int u = 0; u < NB; ++u) {
        const int q = (wave * NB + u) * 64 + lane;
        const int row = q / CH, slot = q % CH;
        const int c = slot ^ ((row >> SH) & (CH - 1));
        int j = n0 + row;
        j = j < p.ncols ? j : 0;                                 // columns past the end compute garbage that is never stored
        const int n = (int)fastdiv((uint32_t)j, p.div_plane);
        const int rem = j - n * (p.OH * p.OW);
        const int oh = (int)fastdiv((uint32_t)rem, p.div_ow);
        const int ow = rem - oh * p.OW;
        boff[u] = (unsigned)(n * p.n_bytes + (oh * p.mul * p.Wp + ow * p.mul) * 32 + (c >> 1) * p.cb_bytes + (c & 1) * 16);
    }
    // --- filter loads: linear
    const unsigned aoff = (unsigned)((wave * NA * 64 + lane) * 16);

    const int step_begin = ks * p.steps_per_split;
    const int nsteps = min(p.cblocks * p.R * p.S - step_begin, p.steps_per_split);
    const size_t a_step_bytes = (size_t)p.Mpad * RB;
    const char *a_base = static_cast<const char *>(p.At) + (size_t)step_begin * a_step_bytes + (size_t)m0 * RB;
    // next step to load: channel block, tap
    int r, s, cb;
    {
        cb = (int)fastdiv((uint32_t)step_begin, p.div_rs);
        const int rs = step_begin - cb * (p.R * p.S);
        r = (int)fastdiv((uint32_t)rs, p.div_s);
        s = rs - r * p.S;
    }
    // The NL loads of a step are issued one at a time (load_one), spread between the matrix instructions: a wave
    // that issues them in a burst stalls on the full memory queue, and with it its matrix pipe.
    const char *xs = nullptr;        // activation base of the step being loaded (tap and channel block applied)
    unsigned la = 0, lb = 0;         // LDS addresses of that step's filter / activation rows of this wave
    auto begin_step_loads = [&](int buf) {
        const int ar = p.sign > 0 ? r : p.R - 1 - r, as = p.sign > 0 ? s : p.S - 1 - s;
        xs = static_cast<const char *>(p.xb) + (size_t)cb * (KC / 16) * p.cb_bytes + (ar * p.Wp + as) * 32;
        la = lds_base + buf * BUF + wave * NA * 1024;
        lb = lds_base + buf * BUF + BM * RB + wave * NB * 1024;
    };
    auto load_one = [&](int i) {     // i < NL, compile-time after unrolling
        if (i < NA) dma16(a_base, aoff + i * 1024, la + i * 1024);
        else dma16(xs, boff[i - NA], lb + (i - NA) * 1024);
    };
    auto end_step_loads = [&]() {
        a_base += a_step_bytes;
        s += 1;
        if (s == p.S) { s = 0; r += 1; }
        if (r == p.R) { r = 0; cb += 1; }
    };
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

    // fragment addresses: row l32 of a 32-row block, chunk (2t + half) ^ swz(row); swz depends on l32 only
    const int l32 = lane & 31, half = lane >> 5;
    const int swzl = (l32 >> SH) & (CH - 1);
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

    // One step.  Slices t = 0 .. NK-1 of 16 channels; the fragments of slice t + 1 are read while slice t is
    // multiplied.  The loads of step + 2 are issued during slices 0 .. NK-2.  Before the LAST slice is multiplied:
    // wait for this wave's loads of step + 1 and for its outstanding fragment reads, barrier, then read slice 0 of
    // step + 1 -- its latency passes under the last slice's matrix instructions.
    constexpr int MPS = TM * TN;                       // matrix instructions per slice
    constexpr int SLOTS = (NK - 1) * MPS;              // ... in the slices that carry loads
    constexpr int SPACING = SLOTS / NL > 0 ? SLOTS / NL : 1;
    static_assert(NL <= SLOTS, "one load per matrix instruction at most");
    int step = 0;
    auto do_step = [&](auto more_c) {                  // more: the loads of step + 2 exist (compile-time)
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
                    const int m = t * MPS + i * TN + jn;           // index among the step's matrix instructions
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
        if (p.ksplit == 1 && p.out_bf16 && p.dst_small && m0 + BM <= p.M && n0 + BN <= p.ncols) {
            // Whole tile inside the tensor: neighbouring lanes (positions col, col + 1 of one sample) trade a value
            // so that the even lane stores row a of both positions and the odd lane row a + 1 of both: one 4-byte
            // store per lane for two accumulator registers, rounded in hardware.  Lanes whose neighbour belongs to
            // another sample store their values one by one.
            typedef float f32x2 __attribute__((ext_vector_type(2)));
            typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
            char *const yb = static_cast<char *>(p.dst);
            const bool odd = l32 & 1;
            const bool pair = odd ? rem >= 1 : rem + 1 < plane;
            const unsigned own = (unsigned)n * (unsigned)p.dst_bs + (unsigned)rem;
            const unsigned row_bytes = 2u * (unsigned)plane;
            const unsigned rowb = (unsigned)(m0 + wm * TM * 32 + half * 4);
            if (pair) {
                const unsigned ob = 2u * (own - (odd ? 1u : 0u)) + (rowb + (odd ? 1u : 0u)) * row_bytes;
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int v = 0; v < 16; v += 2) {
                        const float va = acc[i][jn][v], vb = acc[i][jn][v + 1];
                        const float send = odd ? va : vb;
                        const float recv = __builtin_bit_cast(
                            float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, send), 0xB1, 0xF, 0xF, true));
                        const f32x2 pr = {odd ? recv : va, odd ? vb : recv};
                        const bf16x2 pk = __builtin_convertvector(pr, bf16x2);
                        __builtin_memcpy(yb + (ob + (unsigned)(i * 32 + (v >> 2) * 8 + (v & 3)) * row_bytes), &pk, 4);
                    }
            } else {
                const unsigned ob = 2u * own + rowb * row_bytes;
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const __bf16 r = (__bf16)acc[i][jn][v];
                        __builtin_memcpy(yb + (ob + (unsigned)(i * 32 + (v >> 2) * 8 + (v & 3)) * row_bytes), &r, 2);
                    }
            }
            continue;
        }
        if (p.ksplit == 1 && p.out_bf16) {
            unsigned short *out = static_cast<unsigned short *>(p.dst) + (size_t)n * p.dst_bs + rem;
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
                                  : static_cast<float *>(p.dst) + (size_t)n * p.dst_bs + rem;
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

// One launch prepares both operands of colgemm_bf16_dma_kernel.
//   blocks [0, xb_blocks): xb[n][cb][hp][wp][16] from NCHW bf16 src (samples src_bs elements apart), zeros in the
//                          padding; one thread per (n, cb, hp, wp)
//   the rest:              wt[step][Mpad][kc] from KCRS filters, chunks swizzled; one thread per 8-channel chunk
struct DmaPrepArgs {
    const unsigned short *src;
    u32x4 *xb;
    int N, CB, LH, LW, Hp, Wp, pad_h, pad_w;   // pad_h / pad_w: zero rows above / zero columns left of the data
    int64_t src_bs;
    int xb_blocks;
    int xb_planes;         // 1: block b < xb_blocks stages the 16 planes of (n, cb) = b in LDS (needs 16-byte aligned plane
                           // groups and 32 * LH * LW bytes of dynamic LDS); 0: one thread per position, 2-byte gathers
    const unsigned short *w;
    unsigned short *wt;
    int M, Mpad, cblocks, RS, C, transposed, kc;
    FastDiv div_wp, div_hp, div_cb;
};

__global__ __launch_bounds__(256) void bf16_dma_prepare(const DmaPrepArgs p)
{
    if ((int)blockIdx.x < p.xb_blocks && p.xb_planes) {
        // the 16 planes of one (sample, channel block) are one contiguous run of 32 * LH * LW bytes: copy it into LDS
        // with 16-byte pieces, then every thread gathers the 16 channels of a padded position from LDS
        extern __shared__ __attribute__((aligned(16))) unsigned short planes[];
        const int LHW = p.LH * p.LW;
        const uint32_t n = fastdiv((uint32_t)blockIdx.x, p.div_cb);
        const int cb = (int)(blockIdx.x - n * (uint32_t)p.CB);
        const u32x4 *src = reinterpret_cast<const u32x4 *>(p.src + n * p.src_bs + (int64_t)cb * 16 * LHW);
        for (int v = threadIdx.x; v < 2 * LHW; v += 256) reinterpret_cast<u32x4 *>(planes)[v] = src[v];
        __syncthreads();
        const int PP = p.Hp * p.Wp;
        u32x4 *dst = p.xb + (int64_t)blockIdx.x * PP * 2;
        for (int t = threadIdx.x; t < PP; t += 256) {
            const int hp = (int)fastdiv((uint32_t)t, p.div_wp), wp = t - hp * p.Wp;
            const int h = hp - p.pad_h, w = wp - p.pad_w;
            u32x4 lo = {0u, 0u, 0u, 0u}, hi = {0u, 0u, 0u, 0u};
            if ((unsigned)h < (unsigned)p.LH && (unsigned)w < (unsigned)p.LW) {
                const unsigned short *s = planes + h * p.LW + w;
                unsigned short v[16];
#pragma unroll
                for (int k = 0; k < 16; ++k) v[k] = s[k * LHW];
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    lo[k] = (unsigned)v[2 * k] | ((unsigned)v[2 * k + 1] << 16);
                    hi[k] = (unsigned)v[8 + 2 * k] | ((unsigned)v[8 + 2 * k + 1] << 16);
                }
            }
            dst[2 * t] = lo;
            dst[2 * t + 1] = hi;
        }
        return;
    }
    if ((int)blockIdx.x < p.xb_blocks) {
        const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
        const int64_t total = (int64_t)p.N * p.CB * p.Hp * p.Wp;
        if (i >= total) return;
        const uint32_t t1 = fastdiv((uint32_t)i, p.div_wp);          // (n*CB + cb)*Hp + hp
        const int wp = (int)((uint32_t)i - t1 * (uint32_t)p.Wp);
        const uint32_t t2 = fastdiv(t1, p.div_hp);                    // n*CB + cb
        const int hp = (int)(t1 - t2 * (uint32_t)p.Hp);
        const uint32_t n = fastdiv(t2, p.div_cb);
        const int cb = (int)(t2 - n * (uint32_t)p.CB);
        const int h = hp - p.pad_h, w = wp - p.pad_w;
        u32x4 lo = {0u, 0u, 0u, 0u}, hi = {0u, 0u, 0u, 0u};
        if ((unsigned)h < (unsigned)p.LH && (unsigned)w < (unsigned)p.LW) {
            const int LHW = p.LH * p.LW;
            const unsigned short *s = p.src + n * p.src_bs + (int64_t)cb * 16 * LHW + h * p.LW + w;
            unsigned short v[16];
#pragma unroll
            for (int k = 0; k < 16; ++k) v[k] = s[(int64_t)k * LHW];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                lo[k] = (unsigned)v[2 * k] | ((unsigned)v[2 * k + 1] << 16);
                hi[k] = (unsigned)v[8 + 2 * k] | ((unsigned)v[8 + 2 * k + 1] << 16);
            }
        }
        p.xb[2 * i] = lo;
        p.xb[2 * i + 1] = hi;
        return;
    }
    // filters: one thread per 16-byte chunk (8 consecutive channels of one row and tap)
    const int chunks = p.kc / 8, sh = p.kc == 64 ? 1 : 2;
    int64_t i = (int64_t)(blockIdx.x - p.xb_blocks) * 256 + threadIdx.x;
    const int64_t total = (int64_t)p.cblocks * p.RS * p.Mpad * chunks;
    if (i >= total) return;
    const int c = (int)(i % chunks);
    int64_t t = i / chunks;
    const int m = (int)(t % p.Mpad);
    t /= p.Mpad;
    const int rs = (int)(t % p.RS);
    const int cbk = (int)(t / p.RS);
    const int ch0 = cbk * p.kc + c * 8;
    unsigned short v[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        const int ch = ch0 + k;
        v[k] = m < p.M ? (p.transposed ? p.w[((int64_t)ch * p.C + m) * p.RS + rs] : p.w[((int64_t)m * p.C + ch) * p.RS + rs])
                       : (unsigned short)0;
    }
    const u32x4 o = {(unsigned)v[0] | ((unsigned)v[1] << 16), (unsigned)v[2] | ((unsigned)v[3] << 16),
                     (unsigned)v[4] | ((unsigned)v[5] << 16), (unsigned)v[6] | ((unsigned)v[7] << 16)};
    const int pos = c ^ ((m >> sh) & (chunks - 1));
    reinterpret_cast<u32x4 *>(p.wt)[(i - c) + pos] = o;
}

// ---------------------------------------------------------------------------
// Forward pass of a few-channel layer with bf16 inputs (the 11x11 stride-4 first layer) on
// v_mfma_f32_32x32x16_bf16.  The reduction runs over (c, r) with the filter columns s inside, padded to 16: one
// matrix instruction covers one filter ROW of one channel, and the eight consecutive s a lane feeds are eight
// consecutive bf16 of a staged input row -- two aligned 8-byte LDS reads, no per-element gathers (the padding
// s = S .. 15 multiplies real neighbouring pixels by zero filter entries).  45 % of the matrix work is that
// padding, at a sixteenth of the fp32 instruction cost per product.
//
// Work-groups are persistent: the whole filter bank (C*R slices of [Mpad][16] bf16, 99 KB for 96 filters of
// 3 x 11 x 11) stays in LDS, so the loop over a tile's slices has no barrier; a work-group walks over tiles of
// 128 * TN output positions of one image (a wave owns 32 * TN of them, so that a filter fragment read from LDS feeds
// TN matrix instructions), staging each tile's input rows (zero padding in place) as in colgemm_patch_kernel.  The
// global loads of the next tile's rows are issued before the current tile is multiplied and written to LDS after it.
// Needs: S <= 16, stride % 4 == 0, pad even, W % 8 == 0, batch stride % 8 == 0 (16-byte row loads, 8-byte aligned
// fragment reads).
// ---------------------------------------------------------------------------
struct PatchBf16Args {
    const void *Ft;       // filters [slice = c*R + r][Mpad][16 s] bf16, 8-element halves swapped where (row >> 3) & 1
    const unsigned short *x;
    void *y;              // fp32 or bfloat16 (the kernel's TO)
    int M, Mpad, nslices;
    int C, H, W, R, stride, pad;
    int P, Q, PQ;
    int NR, WP;           // staged rows per channel, LDS row pitch in elements (multiple of 4)
    int x_bs, y_bs;
    int jtiles, ntiles;   // position tiles per image, tiles in all
    int epi_on;
    Epilogue epi;
    FastDiv div_q, div_j, div_nr, div_wv;
};

constexpr int kPatchBf16Pieces(int tn) { return tn == 1 ? 8 : 12; }   // 16-byte row pieces per thread and tile

template <int TM, int TN, typename TO>
__global__ __launch_bounds__(kThreads, 1) void conv_patch_bf16_kernel(const PatchBf16Args p)
{
    constexpr int NV = kPatchBf16Pieces(TN);     // (the host checks the bound)
    constexpr int BN = 128 * TN;                 // positions per tile: 32 * TN per wave
    extern __shared__ __attribute__((aligned(16))) float lds_fast[];
    char *const fl = reinterpret_cast<char *>(lds_fast);                  // filters: nslices * Mpad * 32 bytes
    const int fbytes = p.nslices * p.Mpad * 32;
    unsigned short *const patch = reinterpret_cast<unsigned short *>(fl + fbytes);   // C * NR * WP elements
    const unsigned lds_base = (unsigned)(size_t)lds_fast;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = uniform(tid >> 6);
    const int l32 = lane & 31, half = lane >> 5;

    // filters: linear copy into LDS, 1 KB per wavefront load
    for (int off = wave * 1024; off < fbytes; off += 4 * 1024)
        if (off + lane * 16 < fbytes) dma16(p.Ft, (unsigned)(off + lane * 16), lds_base + off);
    // patch: zero once (the padding columns stay zero for every tile)
    const int pwords = p.C * p.NR * p.WP / 2;
    for (int i = tid; i < pwords; i += kThreads) reinterpret_cast<unsigned *>(patch)[i] = 0u;

    // this lane's bias values, once: accumulator element v of block i belongs to row i*32 + half*4 + (v>>2)*8 + (v&3)
    float bias[TM][16];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v)
            bias[i][v] = (p.epi_on && p.epi.bias) ? p.epi.bias[min(i * 32 + half * 4 + (v >> 2) * 8 + (v & 3), p.M - 1)] : 0.f;

    // This thread's 16-byte pieces of a tile's rows; which piece of which row of which channel does not depend on
    // the tile: piece e = tid + u * kThreads is piece v of staged row i of channel c.
    const int wv = p.W / 8;                      // 16-byte pieces per input row
    const int pieces = p.C * p.NR * wv;
    int prow[NV];                                // staged row i, or a row no tile has (-NR - H) for e >= pieces
    int pgoff[NV];                               // (c*H + i)*W + 8v: element offset in the image at h0 = 0
    int pdst[NV];                                // element offset in the patch: (c*NR + i)*WP + pad + 8v (4-byte aligned)
#pragma unroll
    for (int u = 0; u < NV; ++u) {
        const int e = tid + u * kThreads;
        const int ee = e < pieces ? e : 0;
        const int row = (int)fastdiv((uint32_t)ee, p.div_wv);            // c * NR + i
        const int v = ee - row * wv;
        const int c = (int)fastdiv((uint32_t)row, p.div_nr);
        const int i = row - c * p.NR;
        prow[u] = e < pieces ? i : -p.NR - p.H;
        pgoff[u] = (c * p.H + i) * p.W + v * 8;
        pdst[u] = row * p.WP + p.pad + v * 8;
    }
    u32x4 stage[NV];
    auto first_row = [&](int tile) {             // input row of a tile's staged row 0
        const int n = (int)fastdiv((uint32_t)tile, p.div_j);
        const int p0 = (int)fastdiv((uint32_t)((tile - n * p.jtiles) * BN), p.div_q);
        return p0 * p.stride - p.pad;
    };
    // global loads of a tile's rows into registers; rows outside the image are loaded from a valid address and
    // replaced by zeros only when they are stored (a select on the loaded value here would wait for the load)
    auto load_tile = [&](int tile) {
        const int n = (int)fastdiv((uint32_t)tile, p.div_j);
        const int h0 = first_row(tile);
        const unsigned short *xn = p.x + (size_t)n * p.x_bs + h0 * p.W;
#pragma unroll
        for (int u = 0; u < NV; ++u) {
            const bool ok = (unsigned)(h0 + prow[u]) < (unsigned)p.H;
            stage[u] = *reinterpret_cast<const u32x4 *>(ok ? xn + pgoff[u] : p.x);
        }
    };
    // ... and from the registers into the patch
    auto store_tile = [&](int tile) {
        const int h0 = first_row(tile);
#pragma unroll
        for (int u = 0; u < NV; ++u) {
            if (prow[u] >= 0) {
                const bool ok = (unsigned)(h0 + prow[u]) < (unsigned)p.H;
                unsigned *dst = reinterpret_cast<unsigned *>(patch + pdst[u]);
                dst[0] = ok ? stage[u][0] : 0u; dst[1] = ok ? stage[u][1] : 0u;
                dst[2] = ok ? stage[u][2] : 0u; dst[3] = ok ? stage[u][3] : 0u;
            }
        }
    };

    int tile = blockIdx.x;
    if (tile < p.ntiles) load_tile(tile);
    wait_vmcnt<0>();                             // the filter copy (and the first tile's rows) have landed
    __syncthreads();                             // zero fill done before the rows are written over it

    const int a_off = l32 * 32 + ((half ^ ((l32 >> 3) & 1)) * 16);        // this lane's 16 bytes of a 32-row block
    for (; tile < p.ntiles; tile += gridDim.x) {
        store_tile(tile);
        __syncthreads();
        const int next = tile + gridDim.x;
        if (next < p.ntiles) load_tile(next);

        const int n = (int)fastdiv((uint32_t)tile, p.div_j);
        const int jt = tile - n * p.jtiles;
        const int j0 = jt * BN;
        const int p0 = (int)fastdiv((uint32_t)j0, p.div_q);
        const int jw = j0 + wave * (32 * TN) + l32;              // this lane's position in block 0; block b: + 32 b
        int colbase[TN];                         // element offset of this lane's positions inside a channel's rows
#pragma unroll
        for (int b = 0; b < TN; ++b) {
            const int j = jw + 32 * b;
            const int jj = j < p.PQ ? j : j0;
            const int pp = (int)fastdiv((uint32_t)jj, p.div_q);
            const int qq = jj - pp * p.Q;
            colbase[b] = (pp - p0) * p.stride * p.WP + qq * p.stride + 8 * half;
        }
        f32x16 acc[TM][TN];
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int b = 0; b < TN; ++b)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[i][b][v] = 0.f;

        // slices: three sets of fragments, so that the reads of slices sl + 1 and sl + 2 are in flight while slice
        // sl is multiplied (one wave per SIMD: nothing else hides the LDS latency)
        u32x4 fa[3][TM];
        typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
        u32x2 fb[3][TN][2];
        // next slice to read: its index, its filter row, the byte offsets of its filter block (this lane's) and of
        // its first patch row.  With one wave per SIMD every bookkeeping instruction takes an issue slot that the
        // matrix instructions do not hide, so the offsets advance by additions only.
        int nxt = 0, r = 0;
        unsigned a_cur = (unsigned)a_off, b_cur = 0;
        const unsigned a_step = (unsigned)p.Mpad * 32, row_step = (unsigned)p.WP * 2,
                       wrap_step = (unsigned)(p.NR - p.R + 1) * p.WP * 2;
        unsigned colbytes[TN];
#pragma unroll
        for (int b = 0; b < TN; ++b) colbytes[b] = (unsigned)colbase[b] * 2;
        const char *const pb = reinterpret_cast<const char *>(patch);
        // No branch inside the loop (one would make the compiler wait for the fragment reads right after issuing
        // them): past the last slice, that slice is read again instead.
        auto read_into = [&](int set) {
#pragma unroll
            for (int i = 0; i < TM; ++i) fa[set][i] = *reinterpret_cast<const u32x4 *>(fl + a_cur + i * 1024);
#pragma unroll
            for (int b = 0; b < TN; ++b) {
                fb[set][b][0] = *reinterpret_cast<const u32x2 *>(pb + b_cur + colbytes[b]);
                fb[set][b][1] = *reinterpret_cast<const u32x2 *>(pb + b_cur + colbytes[b] + 8);
            }
            const bool more = nxt + 1 < p.nslices;
            const bool wrap = r + 1 == p.R;
            nxt += more ? 1 : 0;
            a_cur += more ? a_step : 0u;
            b_cur += more ? (wrap ? wrap_step : row_step) : 0u;
            r = wrap ? 0 : r + 1;
        };
        auto multiply = [&](int set) {
#pragma unroll
            for (int b = 0; b < TN; ++b) {
                const u32x4 bq = {fb[set][b][0][0], fb[set][b][0][1], fb[set][b][1][0], fb[set][b][1][1]};
#pragma unroll
                for (int i = 0; i < TM; ++i)
                    acc[i][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fa[set][i]),
                                                                        __builtin_bit_cast(bf16x8, bq), acc[i][b], 0, 0, 0);
            }
        };
        read_into(0);
        read_into(1);
        int sl = 0;
        // One phase = the reads of one slice and the matrix instructions of another.  The scheduling directives
        // spread the phase's reads and bookkeeping between its matrix instructions (with one wave per SIMD an
        // instruction issued between two matrix instructions is free, one issued before or after them is not) and
        // keep the phases apart, so that the compiler cannot move a slice's matrix instructions up to its reads.
        auto phase = [&](int rd, int mul) {
            read_into(rd);
            multiply(mul);
#pragma unroll
            for (int k = 0; k < TM * TN; ++k) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);           // one matrix instruction
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);           // one LDS read
                __builtin_amdgcn_sched_group_barrier(0x006, 4, 0);           // scalar / vector bookkeeping
            }
            __builtin_amdgcn_sched_barrier(0);
        };
        for (; sl + 3 <= p.nslices; sl += 3) {
            phase(2, 0);
            phase(0, 1);
            phase(1, 2);
        }
        if (sl < p.nslices) multiply(0);                         // sets 0 and 1 hold slices sl and sl + 1
        if (sl + 1 < p.nslices) multiply(1);

        if (p.epi_on) {                                              // forward only: bias and ReLU, no mask
            if (p.epi.bias) {
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int b = 0; b < TN; ++b)
#pragma unroll
                        for (int v = 0; v < 16; ++v) acc[i][b][v] += bias[i][v];
            }
            if (p.epi.relu) {
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int b = 0; b < TN; ++b)
#pragma unroll
                        for (int v = 0; v < 16; ++v) acc[i][b][v] = acc[i][b][v] > 0.f ? acc[i][b][v] : 0.f;
            }
        }
        bool stored = false;
        if constexpr (sizeof(TO) == 2) {
            // bfloat16 output, every row and position of the tile inside the tensor: neighbouring lanes (positions
            // j, j + 1) trade one value each, so that the even lane stores row a of both positions and the odd lane
            // row a + 1 of both -- one 4-byte store per lane for two accumulator registers, rounded in hardware
            // (byte offsets from the tensor's base in 32 bits, which the host has checked: one vector addition
            // per store instead of a 64-bit one)
            if (p.M == TM * 32 && j0 + BN <= p.PQ) {
                typedef float f32x2 __attribute__((ext_vector_type(2)));
                typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
                const bool odd = l32 & 1;
                char *const yb = static_cast<char *>(p.y);
                const unsigned ob = 2u * ((unsigned)n * (unsigned)p.y_bs + (unsigned)(half * 4 + (odd ? 1 : 0)) * (unsigned)p.PQ +
                                          (unsigned)(jw & ~1));
                const unsigned row_bytes = 2u * (unsigned)p.PQ;
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int b = 0; b < TN; ++b)
#pragma unroll
                        for (int v = 0; v < 16; v += 2) {
                            const float va = acc[i][b][v], vb = acc[i][b][v + 1];
                            const float send = odd ? va : vb;
                            const float recv = __builtin_bit_cast(
                                float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, send), 0xB1, 0xF, 0xF, true));
                            const f32x2 pr = {odd ? recv : va, odd ? vb : recv};
                            const bf16x2 pk = __builtin_convertvector(pr, bf16x2);
                            __builtin_memcpy(yb + (ob + (unsigned)(i * 32 + (v >> 2) * 8 + (v & 3)) * row_bytes + 64u * b), &pk, 4);
                        }
                stored = true;
            }
        }
        if (!stored) {
#pragma unroll
            for (int b = 0; b < TN; ++b) {
                const int j = jw + 32 * b;
                if (j < p.PQ) {
                    TO *out = static_cast<TO *>(p.y) + (size_t)n * p.y_bs + j;
#pragma unroll
                    for (int i = 0; i < TM; ++i)
#pragma unroll
                        for (int v = 0; v < 16; ++v) {
                            const int row = i * 32 + half * 4 + (v >> 2) * 8 + (v & 3);
                            if (row < p.M) st_elem(out, (int64_t)row * p.PQ, acc[i][b][v]);
                        }
                }
            }
        }
        wait_vmcnt<0>();                         // next tile's rows are in the registers
        __syncthreads();                         // every wave is done reading this tile's patch
    }
}

// Filters for conv_patch_bf16_kernel: Ft[c*R + r][Mpad][16] bf16 from w[k][c][r][s]; zeros for s >= S and rows >= M;
// the two 8-element halves of a row swapped where (row >> 3) & 1 (bank spread of the fragment reads)
__global__ void relayout_filters_rows_bf16(const unsigned short *__restrict__ w, unsigned short *__restrict__ ft,
                                           int M, int Mpad, int C, int R, int S)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t total = (int64_t)C * R * Mpad * 16;
    if (i >= total) return;
    const int s = (int)(i & 15);
    int64_t t = i >> 4;
    const int m = (int)(t % Mpad);
    const int sl = (int)(t / Mpad);
    const int c = sl / R, r = sl - c * R;
    unsigned short v = 0;
    if (m < M && s < S) v = w[(((int64_t)m * C + c) * R + r) * S + s];
    const int pos = (s >> 3) ^ ((m >> 3) & 1);
    ft[(i - s) + pos * 8 + (s & 7)] = v;
}
